"""Pins of the CPU oracle against things other than itself.

Each pin is chosen so that a plausible mistake in oracle/moe_oracle.py (a dropped
term, a wrong sign or index, a transposed operand) fails at least one of them:
  1. hand-worked closed forms (tests/golden/*.txt);
  2. invariants BASELINE's north star names (counts sum to T*k, weights sum to 1,
     the permutation is a bijection), on all five workload shapes;
  3. the dense all-experts-masked evaluation of Eq. 3, differentiated by torch autograd;
  4. central finite differences of the oracle's own forward pass;
  5. special cases that reduce to plain matrix products or library routines.
The last test plants mistakes into the oracle and checks that the pins notice.
"""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import moe_oracle as orc

from .helpers import (np64, oracle_inputs, problem, read_route_golden, read_swiglu_golden,
                      scale_rel_err, small_cfg)


# ------------------------------------------------------------------ 1. closed forms
@pytest.mark.parametrize("case", read_route_golden(), ids=lambda c: f"{c[0]}-r{int(c[1])}-k{c[2]}")
def test_route_closed_forms(case):
    gate, renorm, k, logits, idx_exp, w_exp = case
    lg = np.array([logits], dtype=np.float32)
    idx, w = orc.route(lg, k, gate, renorm)
    assert idx.dtype == np.int32
    assert idx[0].tolist() == idx_exp
    # logits pass through fp32, so exp(log a) carries ~1e-7 relative error
    np.testing.assert_allclose(w[0], w_exp, rtol=5e-7)


def test_swiglu_closed_form():
    g = read_swiglu_golden()
    G, U, H, Y = orc.swiglu_ffn(g["x"], g["Wg"], g["Wu"], g["Wd"])
    for got, name in ((G, "g"), (U, "u"), (H, "h"), (Y, "y")):
        np.testing.assert_allclose(got, g[name], rtol=1e-13, atol=1e-14)
    dx, dWg, dWu, dWd, dg, du = orc.swiglu_ffn_bwd(g["x"], g["Wg"], g["Wu"], g["Wd"], G, U, g["dy"])
    for got, name in ((dx, "dx"), (dWg, "dWg"), (dWu, "dWu"), (dWd, "dWd"), (dg, "dg"), (du, "du")):
        np.testing.assert_allclose(got, g[name], rtol=1e-13, atol=1e-14)


def test_dispatch_worked_example():
    # 4 tokens, k=2, E=4.  Assignments a=0..7 go to experts 2,0 | 0,3 | 2,3 | 0,2.
    idx = np.array([[2, 0], [0, 3], [2, 3], [0, 2]], dtype=np.int32)
    counts, offsets, row_of, src_of = orc.dispatch_plan(idx, 4)
    assert counts.tolist() == [3, 0, 3, 2]
    assert offsets.tolist() == [0, 3, 3, 6, 8]
    # expert 0 gets a=1,2,6 (rows 0,1,2); expert 2 gets a=0,4,7 (rows 3,4,5); expert 3 gets a=3,5 (rows 6,7)
    assert row_of.tolist() == [3, 0, 1, 6, 4, 7, 2, 5]
    assert src_of.tolist() == [1, 2, 6, 0, 4, 7, 3, 5]
    ids, n = orc.active_experts(counts)
    assert int(n) == 3 and ids.tolist() == [0, 2, 3, -1]
    X = np.arange(8, dtype=np.float64).reshape(4, 2)
    Xp = orc.permute_rows(X, row_of, 2)
    assert Xp[:, 0].tolist() == [0, 2, 6, 0, 4, 6, 2, 4]  # token ids 0,1,3 | 0,2,3 | 1,2 times 2
    # combine with weights: Y[t] = sum_j w[t,j] * Yp[row_of[t*2+j]]
    Yp = np.arange(8, dtype=np.float64).reshape(8, 1) + 1.0  # row r holds r+1
    w = np.array([[0.5, 0.5], [1.0, 0.0], [0.25, 0.75], [2.0, 1.0]])
    Y = orc.combine(Yp, row_of, w)
    assert Y[:, 0].tolist() == [0.5 * 4 + 0.5 * 1, 2.0, 0.25 * 5 + 0.75 * 8, 2.0 * 3 + 6.0]
    dYp, dw = orc.combine_bwd(np.array([[1.0], [2.0], [3.0], [4.0]]), Yp, row_of, w)
    assert dw.tolist() == [[4.0, 1.0], [4.0, 14.0], [15.0, 24.0], [12.0, 24.0]]
    assert dYp[:, 0].tolist() == [0.5, 2.0, 8.0, 0.5, 0.75, 4.0, 0.0, 2.25]


# --------------------------------------------------------------------- 2. invariants
@pytest.mark.parametrize("name", list(wl.CONFIGS))
def test_routing_invariants_all_configs(name):
    cfg = wl.CONFIGS[name]
    logits = wl.make_logits(cfg).numpy()
    idx, w = orc.route(logits, cfg.k, cfg.gate, cfg.renorm)
    counts, offsets, row_of, src_of = orc.dispatch_plan(idx, cfg.E)
    A = cfg.T * cfg.k
    assert int(counts.sum()) == A                      # no token dropped
    assert offsets[0] == 0 and offsets[-1] == A
    assert np.all(np.diff(offsets) == counts)
    assert np.array_equal(np.sort(row_of), np.arange(A))  # bijection
    assert np.array_equal(src_of[row_of], np.arange(A))
    assert idx.min() >= 0 and idx.max() < cfg.E
    srt = np.sort(idx, axis=1)
    assert np.all(srt[:, 1:] != srt[:, :-1])            # k distinct experts per token
    np.testing.assert_allclose(w.sum(axis=1), 1.0, atol=1e-12)
    assert np.all(w > 0) and np.all(w[:, :-1] >= w[:, 1:])
    # library routines as the reference of the integer outputs
    flat = idx.reshape(-1)
    assert np.array_equal(counts, np.bincount(flat, minlength=cfg.E))
    assert np.array_equal(src_of, np.argsort(flat, kind="stable"))
    # rows of one expert are in ascending assignment order
    e_of_row = flat[src_of]
    assert np.all(np.diff(e_of_row) >= 0)
    same = e_of_row[1:] == e_of_row[:-1]
    assert np.all(np.diff(src_of)[same] > 0)
    # selection against torch.topk where the k-th and (k+1)-th logits differ
    tk = torch.topk(torch.from_numpy(logits), cfg.k, dim=1).indices.numpy()
    assert np.array_equal(np.sort(tk, axis=1), srt)
    ids, n = orc.active_experts(counts)
    assert int(n) == int((counts > 0).sum())
    assert np.all(counts[ids[:int(n)]] > 0) and np.all(np.diff(ids[:int(n)]) > 0)
    if cfg.routing == "stress":
        hot, zero, n_hot = wl.stress_sets(cfg)
        assert counts[hot] == n_hot == 4915
        assert np.all(counts[zero] == 0)


# ------------------------------------------------- 3. dense masked Eq. 3 + autograd
def dense_masked_autograd(p, cfg, w_leaf=None):
    """Eq. 3 with every expert run on every token and a 0/1 mask; gradients by autograd.

    If w_leaf is given ([T,k] weights and the selected indices) it replaces the gate, so
    the gradient with respect to the combine weights can be read off.
    """
    t64 = lambda a: torch.tensor(np64(a), dtype=torch.float64, requires_grad=True)
    X, Wg, Wu, Wd = t64(p["X"]), t64(p["Wg"]), t64(p["Wu"]), t64(p["Wd"])
    logits = torch.tensor(np64(p["logits"]), dtype=torch.float64, requires_grad=True)
    leaves = {"X": X, "Wg": Wg, "Wu": Wu, "Wd": Wd, "logits": logits}
    T, E = logits.shape
    if w_leaf is None:
        s = torch.softmax(logits, 1) if cfg.gate == "softmax" else torch.sigmoid(logits)
        sel = torch.topk(torch.tensor(p["logits"].numpy()), cfg.k, dim=1).indices
        mask = torch.zeros(T, E, dtype=torch.float64).scatter_(1, sel, 1.0)
        wfull = s * mask
        if cfg.renorm:
            wfull = wfull / wfull.sum(1, keepdim=True)
    else:
        wsel, idx = w_leaf
        wsel = torch.tensor(wsel, dtype=torch.float64, requires_grad=True)
        leaves["w"] = wsel
        wfull = torch.zeros(T, E, dtype=torch.float64).scatter(1, torch.tensor(idx, dtype=torch.int64), wsel)
    Y = torch.zeros_like(X)
    for e in range(E):
        h = torch.nn.functional.silu(X @ Wg[e]) * (X @ Wu[e])
        Y = Y + wfull[:, e:e + 1] * (h @ Wd[e])
    if cfg.n_shared:
        Wsg, Wsu, Wsd = t64(p["Wsg"]), t64(p["Wsu"]), t64(p["Wsd"])
        leaves.update(Wsg=Wsg, Wsu=Wsu, Wsd=Wsd)
        for s_ in range(cfg.n_shared):
            Y = Y + (torch.nn.functional.silu(X @ Wsg[s_]) * (X @ Wsu[s_])) @ Wsd[s_]
    loss = (Y * torch.tensor(np64(p["dY"]))).sum()
    loss.backward()
    grads = {"d" + n: v.grad.numpy() for n, v in leaves.items() if v.grad is not None}
    return Y.detach().numpy(), grads, wfull.detach().numpy()


def run_oracle(p, cfg, **kw):
    o = oracle_inputs(p)
    return orc.layer_fwd_bwd(o["logits"], o["X"], o["dY"], o["Wg"], o["Wu"], o["Wd"], cfg.k, cfg.gate, cfg.renorm,
                             o.get("Wsg"), o.get("Wsu"), o.get("Wsd"), want_dlogits=True, **kw)


BRUTE = [
    small_cfg(T=24, d=8, E=6, k=2, d_ff=12),
    small_cfg(T=32, d=16, E=8, k=3, d_ff=10, gate="sigmoid"),
    small_cfg(T=20, d=8, E=5, k=2, d_ff=6, renorm=False),
    small_cfg(T=20, d=8, E=5, k=2, d_ff=6, renorm=False, gate="sigmoid"),
    small_cfg(T=16, d=8, E=8, k=4, d_ff=8, n_shared=2, d_ff_shared=6, zipf_s=2.0),
    small_cfg(T=12, d=4, E=4, k=1, d_ff=4),
]


@pytest.mark.parametrize("cfg", BRUTE, ids=lambda c: f"T{c.T}E{c.E}k{c.k}{c.gate}{int(c.renorm)}s{c.n_shared}")
def test_dense_masked_brute_force_and_autograd(cfg):
    p = problem(cfg)
    o = run_oracle(p, cfg)
    Y, g, wfull = dense_masked_autograd(p, cfg)
    tol = dict(rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(o["Y"], Y, **tol)
    # combine weights scattered to [T,E] equal the dense masked weights
    wo = np.zeros_like(wfull)
    np.put_along_axis(wo, o["topk_idx"].astype(np.int64), o["topk_w"], axis=1)
    np.testing.assert_allclose(wo, wfull, **tol)
    np.testing.assert_allclose(o["dX"], g["dX"], **tol)
    np.testing.assert_allclose(o["dWg"], g["dWg"], **tol)
    np.testing.assert_allclose(o["dWu"], g["dWu"], **tol)
    np.testing.assert_allclose(o["dWd"], g["dWd"], **tol)
    np.testing.assert_allclose(o["dlogits"], g["dlogits"], **tol)
    if cfg.n_shared:
        for n in ("dWsg", "dWsu", "dWsd"):
            np.testing.assert_allclose(o[n], g[n], **tol)
    # gradient with respect to the combine weights themselves
    _, g2, _ = dense_masked_autograd(p, cfg, w_leaf=(o["topk_w"], o["topk_idx"]))
    np.testing.assert_allclose(o["dw"], g2["dw"], **tol)
    # experts without rows have exactly zero gradient and no slot in the compact buffers
    n_act = int(o["n_active"])
    for e in range(cfg.E):
        if o["counts"][e] == 0:
            assert not o["dWg"][e].any() and not o["dWu"][e].any() and not o["dWd"][e].any()
    c = orc.compact(o["dWg"], o["active_ids"], n_act)
    assert c.shape[0] == n_act
    for i in range(n_act):
        assert np.array_equal(c[i], o["dWg"][o["active_ids"][i]])


# ------------------------------------------------------------ 4. finite differences
def test_finite_differences():
    cfg = small_cfg(T=16, d=8, E=4, k=2, d_ff=12, n_shared=1, d_ff_shared=5)
    p = problem(cfg)
    o = run_oracle(p, cfg)
    base = oracle_inputs(p)

    def loss(inp, w=None):
        idx, ww = orc.route(inp["logits"], cfg.k, cfg.gate, cfg.renorm)
        assert np.array_equal(idx, o["topk_idx"])
        ww = ww if w is None else w
        _, _, row_of, _ = orc.dispatch_plan(idx, cfg.E)[0:4]
        Xp = orc.permute_rows(inp["X"], row_of, cfg.k)
        offsets = orc.dispatch_plan(idx, cfg.E)[1]
        Yp = orc.expert_fwd(Xp, offsets, inp["Wg"], inp["Wu"], inp["Wd"])[3]
        Ysh = orc.shared_fwd(inp["X"], inp["Wsg"], inp["Wsu"], inp["Wsd"])[2]
        return float((orc.combine(Yp, row_of, ww, Ysh) * inp["dY"]).sum())

    rng = np.random.default_rng(0)
    names = {"X": "dX", "Wg": "dWg", "Wu": "dWu", "Wd": "dWd", "Wsg": "dWsg", "Wsu": "dWsu", "Wsd": "dWsd"}
    for name, gname in names.items():
        arr = base[name]
        h = 1e-5 * max(1.0, float(np.abs(arr).max()))
        for _ in range(12):
            pos = tuple(int(rng.integers(0, s)) for s in arr.shape)
            if gname in ("dWg", "dWu", "dWd") and o["counts"][pos[0]] == 0:
                continue
            plus = {k: v.copy() for k, v in base.items()}
            minus = {k: v.copy() for k, v in base.items()}
            plus[name][pos] += h
            minus[name][pos] -= h
            fd = (loss(plus) - loss(minus)) / (2 * h)
            an = o[gname][pos]
            assert abs(fd - an) <= 1e-6 * max(1.0, abs(an)), (name, pos, fd, an)
    # with respect to the combine weights (selection untouched)
    for _ in range(12):
        pos = (int(rng.integers(0, cfg.T)), int(rng.integers(0, cfg.k)))
        wp, wm = o["topk_w"].copy(), o["topk_w"].copy()
        wp[pos] += 1e-6
        wm[pos] -= 1e-6
        fd = (loss(base, wp) - loss(base, wm)) / 2e-6
        assert abs(fd - o["dw"][pos]) <= 1e-6 * max(1.0, abs(o["dw"][pos]))
    # with respect to the logits, where the selection cannot flip
    lg = base["logits"].astype(np.float64)
    srt = np.sort(lg, axis=1)[:, ::-1]
    safe = np.where(srt[:, cfg.k - 1] - srt[:, cfg.k] > 1e-2)[0]
    assert len(safe) > 4
    for t in safe[:8]:
        e = int(rng.integers(0, cfg.E))
        h = 1e-3  # exactly representable steps are not needed: logits are widened before use

        def with_logit(delta):
            inp = dict(base)
            l2 = lg.copy()
            l2[t, e] += delta
            idx = o["topk_idx"]
            s = orc.gate_scores(l2, cfg.gate)
            ww = np.take_along_axis(s, idx.astype(np.int64), axis=1)
            ww = ww / ww.sum(axis=1, keepdims=True)
            return loss(inp, ww)

        fd = (with_logit(h) - with_logit(-h)) / (2 * h)
        assert abs(fd - o["dlogits"][t, e]) <= 1e-5 * max(1.0, abs(o["dlogits"][t, e]))


# ---------------------------------------------------------------- 5. special cases
def torch_ffn(X, Wg, Wu, Wd):
    X, Wg, Wu, Wd = (torch.tensor(np64(a)) for a in (X, Wg, Wu, Wd))
    return ((torch.nn.functional.silu(X @ Wg) * (X @ Wu)) @ Wd).numpy()


def test_single_expert_is_one_ffn():
    cfg = small_cfg(T=10, d=8, E=1, k=1, d_ff=6)
    p = problem(cfg)
    o = run_oracle(p, cfg)
    np.testing.assert_allclose(o["topk_w"], 1.0)
    np.testing.assert_allclose(o["Y"], torch_ffn(p["X"], p["Wg"][0], p["Wu"][0], p["Wd"][0]), rtol=1e-12, atol=1e-14)
    assert np.array_equal(o["row_of"], np.arange(10))


def test_identical_experts_ignore_routing():
    cfg = small_cfg(T=16, d=8, E=6, k=3, d_ff=6)
    p = problem(cfg)
    for n in ("Wg", "Wu", "Wd"):
        p[n] = p[n][:1].expand_as(p[n]).contiguous()
    o = run_oracle(p, cfg)
    np.testing.assert_allclose(o["Y"], torch_ffn(p["X"], p["Wg"][0], p["Wu"][0], p["Wd"][0]), rtol=1e-11, atol=1e-13)


def test_k_equals_E_is_soft_mixture():
    cfg = small_cfg(T=8, d=8, E=4, k=4, d_ff=6)
    p = problem(cfg)
    o = run_oracle(p, cfg)
    s = torch.softmax(torch.tensor(np64(p["logits"])), 1).numpy()
    Y = sum(s[:, e:e + 1] * torch_ffn(p["X"], p["Wg"][e], p["Wu"][e], p["Wd"][e]) for e in range(4))
    np.testing.assert_allclose(o["Y"], Y, rtol=1e-11, atol=1e-13)


def test_expert_relabelling_invariance():
    # placement does not change the result (the paper: total expert computation is unchanged)
    cfg = small_cfg(T=20, d=8, E=6, k=2, d_ff=6)
    p = problem(cfg)
    o = run_oracle(p, cfg)
    perm = torch.tensor([3, 5, 0, 1, 4, 2])
    q = dict(p)
    q["logits"] = p["logits"][:, perm].contiguous()
    for n in ("Wg", "Wu", "Wd"):
        q[n] = p[n][perm].contiguous()
    o2 = run_oracle(q, cfg)
    np.testing.assert_allclose(o2["Y"], o["Y"], rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(o2["dX"], o["dX"], rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(o2["dWg"], o["dWg"][perm.numpy()], rtol=1e-12, atol=1e-14)
    assert np.array_equal(o2["counts"], o["counts"][perm.numpy()])


def test_shared_experts_concatenate_along_dff():
    # Eq. 2: experts summed = one expert with weights concatenated along d_ff
    cfg = small_cfg(T=12, d=8, E=4, k=2, d_ff=6, n_shared=3, d_ff_shared=4)
    p = problem(cfg)
    o = run_oracle(p, cfg)
    cat = dict(p)
    cat["Wsg"] = torch.cat(list(p["Wsg"]), dim=1)[None]
    cat["Wsu"] = torch.cat(list(p["Wsu"]), dim=1)[None]
    cat["Wsd"] = torch.cat(list(p["Wsd"]), dim=0)[None]
    o2 = run_oracle(cat, wl.scaled(cfg, n_shared=1, d_ff_shared=12))
    np.testing.assert_allclose(o2["Y"], o["Y"], rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(o2["dX"], o["dX"], rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(o2["dWsg"][0], np.concatenate(list(o["dWsg"]), axis=1), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(o2["dWsd"][0], np.concatenate(list(o["dWsd"]), axis=0), rtol=1e-12, atol=1e-14)


def test_topk_softmax_equals_softmax_over_selected():
    cfg = small_cfg(T=64, d=8, E=16, k=4, d_ff=4)
    lg = wl.make_logits(cfg).numpy()
    idx, w = orc.route(lg, 4, "softmax", True)
    sel = np.take_along_axis(lg.astype(np.float64), idx.astype(np.int64), axis=1)
    np.testing.assert_allclose(w, torch.softmax(torch.tensor(sel), 1).numpy(), rtol=1e-12)


def test_token_function_matches_layer():
    cfg = small_cfg(T=12, d=8, E=5, k=2, d_ff=6, n_shared=1, d_ff_shared=4)
    p = problem(cfg)
    o = run_oracle(p, cfg)
    q = oracle_inputs(p)
    for t in (0, 5, 11):
        y, dx, dw = orc.token_fwd_bwd(q["X"][t], o["topk_idx"][t], o["topk_w"][t], q["dY"][t], q["Wg"], q["Wu"],
                                      q["Wd"], q["Wsg"], q["Wsu"], q["Wsd"])
        np.testing.assert_allclose(y, o["Y"][t], rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(dx, o["dX"][t], rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(dw, o["dw"][t], rtol=1e-12, atol=1e-14)


def test_fp32_instance_close_to_fp64():
    cfg = wl.scaled(wl.CONFIGS["tiny"], T=64)
    p = problem(cfg, unit_scale=False)
    a = run_oracle(p, cfg)
    b = run_oracle(p, cfg, R=np.float32)
    for n in ("Y", "dX", "dWg", "dWu", "dWd", "dw"):
        assert scale_rel_err(b[n], a[n]) < 1e-5, n
    for n in ("topk_idx", "counts", "offsets", "row_of", "src_of"):
        assert np.array_equal(a[n], b[n])


# ------------------------------------------------- planted mistakes must be noticed
def _pins_pass():
    try:
        test_swiglu_closed_form()
        test_dispatch_worked_example()
        for c in read_route_golden():
            test_route_closed_forms(c)
        test_dense_masked_brute_force_and_autograd(BRUTE[4])
        test_dense_masked_brute_force_and_autograd(BRUTE[1])
        test_dense_masked_brute_force_and_autograd(BRUTE[2])
    except AssertionError:
        return False
    return True


def test_router_linear_map_closed_form_and_autograd():
    """router_fwd / router_bwd: a hand-worked 2x2 case, then torch autograd on a random case."""
    X = np.array([[1.0, 2.0], [-1.0, 0.5]])
    Wr = np.array([[3.0, -1.0, 0.0], [0.5, 2.0, 1.0]])
    np.testing.assert_array_equal(orc.router_fwd(X, Wr), np.array([[4.0, 3.0, 2.0], [-2.75, 2.0, 0.5]]))
    dl = np.array([[1.0, 0.0, -1.0], [2.0, 1.0, 0.0]])
    dX, dWr = orc.router_bwd(X, Wr, dl)
    np.testing.assert_array_equal(dX, np.array([[3.0, -0.5], [5.0, 3.0]]))
    np.testing.assert_array_equal(dWr, np.array([[-1.0, -1.0, -1.0], [3.0, 0.5, -2.0]]))
    rng = np.random.default_rng(3)
    X, Wr, dl = rng.normal(size=(13, 7)), rng.normal(size=(7, 5)), rng.normal(size=(13, 5))
    tx = torch.tensor(X, requires_grad=True)
    tw = torch.tensor(Wr, requires_grad=True)
    lg = tx @ tw
    np.testing.assert_allclose(orc.router_fwd(X, Wr), lg.detach().numpy(), rtol=1e-13, atol=1e-13)
    (lg * torch.tensor(dl)).sum().backward()
    dX, dWr = orc.router_bwd(X, Wr, dl)
    np.testing.assert_allclose(dX, tx.grad.numpy(), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(dWr, tw.grad.numpy(), rtol=1e-12, atol=1e-13)


def test_planted_mistake_in_router_is_caught(monkeypatch):
    real = orc.router_bwd

    def transposed(X, Wr, dlogits, R=np.float64):
        dX, dWr = real(X, Wr, dlogits, R)
        return dX, (np.asarray(dlogits).T @ np.asarray(X)).T[::-1]  # rows of dWr reversed

    with monkeypatch.context() as m:
        m.setattr(orc, "router_bwd", transposed)
        with pytest.raises(AssertionError):
            test_router_linear_map_closed_form_and_autograd()
    test_router_linear_map_closed_form_and_autograd()


def test_planted_mistakes_are_caught(monkeypatch):
    assert _pins_pass()
    real = {n: getattr(orc, n) for n in ("silu", "swiglu_ffn_bwd", "combine", "combine_bwd", "dispatch_plan",
                                         "gate_scores", "select_topk", "route_bwd")}

    def bad_silu(z):  # sign of the exponent
        return z / (1.0 + np.exp(z))

    def bad_bwd_dropped_term(x, Wg, Wu, Wd, g, u, dy):
        sig = 1.0 / (1.0 + np.exp(-g))
        dh = dy @ Wd.T
        du = dh * (g * sig)
        dg = dh * u * sig  # g*(1-sig) term dropped
        return dg @ Wg.T + du @ Wu.T, x.T @ dg, x.T @ du, (g * sig * u).T @ dy, dg, du

    def bad_bwd_swapped(x, Wg, Wu, Wd, g, u, dy):
        dx, a, b, c, dg, du = real["swiglu_ffn_bwd"](x, Wg, Wu, Wd, g, u, dy)
        return dx, b, a, c, dg, du  # dWg and dWu exchanged

    def bad_combine(Yp, row_of, w, Yadd=None, R=np.float64):
        return real["combine"](Yp, row_of, w, None, R)  # shared-expert term dropped

    def bad_combine_bwd(dY, Yp, row_of, w, R=np.float64):
        dYp, dw = real["combine_bwd"](dY, Yp, row_of, w, R)
        return dYp, dw[:, ::-1].copy()  # slot index reversed

    def bad_dispatch(idx, E):
        c, o, r, s = real["dispatch_plan"](idx, E)
        A = r.shape[0]
        r2 = (o[:-1][np.asarray(idx).reshape(-1)] + c[np.asarray(idx).reshape(-1)] - 1
              - (r - o[:-1][np.asarray(idx).reshape(-1)])).astype(np.int32)  # unstable: reversed inside each expert
        s2 = np.empty(A, dtype=np.int32)
        s2[r2] = np.arange(A, dtype=np.int32)
        return c, o, r2, s2

    def bad_gate(logits, gate, R=np.float64):
        return real["gate_scores"](logits, "softmax", R)  # sigmoid ignored

    def bad_topk(logits, k):
        lg = np.asarray(logits)
        return np.argsort(-lg, axis=1, kind="stable")[:, ::-1][:, -k:].astype(np.int32)  # ascending slots

    def bad_route_bwd(logits, idx, dw, gate="softmax", renorm=True, R=np.float64):
        return real["route_bwd"](logits, idx, dw, gate, False, R)  # renormalisation ignored

    plants = {"silu": bad_silu, "swiglu_ffn_bwd": bad_bwd_dropped_term, "combine": bad_combine,
              "combine_bwd": bad_combine_bwd, "dispatch_plan": bad_dispatch, "gate_scores": bad_gate,
              "select_topk": bad_topk, "route_bwd": bad_route_bwd}
    for name, fn in plants.items():
        with monkeypatch.context() as m:
            m.setattr(orc, name, fn)
            assert not _pins_pass(), f"planted mistake in {name} went unnoticed"
    with monkeypatch.context() as m:
        m.setattr(orc, "swiglu_ffn_bwd", bad_bwd_swapped)
        assert not _pins_pass(), "exchanged dWg/dWu went unnoticed"
    assert _pins_pass()


# ------------------------------------------------------------------ auxiliary load-balancing loss
def _aux_pins():
    """Closed forms, a hand-worked case, an independent torch evaluation with autograd, finite
    differences and invariants of aux_loss / aux_loss_bwd."""
    rng = np.random.default_rng(11)
    alpha = 0.001
    for gate in ("softmax", "sigmoid"):
        # uniform scores: L = alpha whatever the loads
        T, E, k = 12, 6, 2
        counts = rng.multinomial(T * k, np.ones(E) / E)
        L, P = orc.aux_loss(np.full((T, E), 0.7), counts, k, alpha, gate)
        np.testing.assert_allclose(L, alpha, rtol=1e-14)
        np.testing.assert_allclose(P, np.full(E, 1.0 / E), rtol=1e-14)
        # uniform loads: L = alpha whatever the scores (the shares of a token sum to one)
        L, P = orc.aux_loss(rng.normal(size=(T, E)), np.full(E, T * k // E), k, alpha, gate)
        np.testing.assert_allclose(L, alpha, rtol=1e-13)
        np.testing.assert_allclose(P.sum(), 1.0, rtol=1e-14)
    # everything on one expert, top-1: L -> alpha * E
    T, E = 5, 4
    lg = np.zeros((T, E))
    lg[:, 2] = 60.0
    L, _ = orc.aux_loss(lg, np.array([0, 0, T, 0]), 1, alpha, "softmax")
    np.testing.assert_allclose(L, alpha * E, rtol=1e-12)
    # hand-worked: 2 tokens, 2 experts, top-1, logits (ln 3, 0) and (0, 0): shares (3/4, 1/4), (1/2, 1/2);
    # P = (5/8, 3/8); counts (2, 0): f = (1, 0); L = alpha * 2 * 5/8
    lg = np.array([[np.log(3.0), 0.0], [0.0, 0.0]])
    L, P = orc.aux_loss(lg, np.array([2, 0]), 1, 1.0, "softmax")
    np.testing.assert_allclose(P, [0.625, 0.375], rtol=1e-15)
    np.testing.assert_allclose(L, 1.25, rtol=1e-15)
    # gradient of that case: c = alpha E f / T = (1, 0); dz_t0 = p0 (1 - p0) = 3/16 and 1/4
    g = orc.aux_loss_bwd(lg, np.array([2, 0]), 1, 1.0, "softmax")
    np.testing.assert_allclose(g, [[3.0 / 16, -3.0 / 16], [0.25, -0.25]], rtol=1e-14)
    # sigmoid gate, same logits: s = (3/4, 1/2), (1/2, 1/2): shares (3/5, 2/5), (1/2, 1/2); P0 = 11/20
    L, P = orc.aux_loss(lg, np.array([2, 0]), 1, 1.0, "sigmoid")
    np.testing.assert_allclose(P, [0.55, 0.45], rtol=1e-15)
    np.testing.assert_allclose(L, 1.1, rtol=1e-15)
    for gate in ("softmax", "sigmoid"):
        T, E, k = 9, 7, 3
        lg = rng.normal(size=(T, E)) * 2.0
        counts = rng.multinomial(T * k, rng.dirichlet(np.ones(E)))
        # independent evaluation in torch, differentiated by autograd
        tz = torch.tensor(lg, requires_grad=True)
        if gate == "softmax":
            tp = torch.softmax(tz, dim=1)
        else:
            ts = torch.sigmoid(tz)
            tp = ts / ts.sum(dim=1, keepdim=True)
        tf = torch.tensor(counts, dtype=torch.float64) / (T * k)
        tL = 0.3 * E * (tf * tp.mean(dim=0)).sum()
        L, _ = orc.aux_loss(lg, counts, k, 0.3, gate)
        np.testing.assert_allclose(L, tL.item(), rtol=1e-13)
        (tL * 1.7).backward()
        g = orc.aux_loss_bwd(lg, counts, k, 0.3, gate, dloss=1.7)
        np.testing.assert_allclose(g, tz.grad.numpy(), rtol=1e-11, atol=1e-15)
        # central finite differences on a few entries
        h = 1e-6
        for (t, e) in ((0, 0), (4, 3), (8, 6)):
            zp, zm = lg.copy(), lg.copy()
            zp[t, e] += h
            zm[t, e] -= h
            fd = (orc.aux_loss(zp, counts, k, 0.3, gate)[0] - orc.aux_loss(zm, counts, k, 0.3, gate)[0]) / (2 * h)
            np.testing.assert_allclose(g[t, e] / 1.7, fd, rtol=1e-6, atol=1e-10)
        if gate == "softmax":  # a shift of a token's logits changes nothing
            np.testing.assert_allclose(g.sum(axis=1), 0.0, atol=1e-15)


def test_aux_loss_pins():
    _aux_pins()


def test_planted_mistakes_in_aux_loss_are_caught(monkeypatch):
    real_loss, real_bwd, real_shares = orc.aux_loss, orc.aux_loss_bwd, orc.gate_shares

    def loss_per_token(logits, counts, k, alpha, gate="softmax", R=np.float64):  # loads divided by T, not T k
        L, P = real_loss(logits, counts, k, alpha, gate, R)
        return L * k, P

    def loss_no_E(logits, counts, k, alpha, gate="softmax", R=np.float64):  # factor E dropped
        L, P = real_loss(logits, counts, k, alpha, gate, R)
        return L / np.asarray(logits).shape[1], P

    def bwd_not_centred(logits, counts, k, alpha, gate="softmax", dloss=1.0, R=np.float64):  # - sum_j p_j c_j dropped
        p = real_shares(logits, gate, R)
        T, E = p.shape
        c = dloss * alpha * E * (np.asarray(counts) / (T * k)) / T
        return p * c[None, :]

    def shares_unnormalised(logits, gate, R=np.float64):  # sigmoid scores not divided by their sum
        return orc.gate_scores(logits, gate, R)

    for name, bad in (("aux_loss", loss_per_token), ("aux_loss", loss_no_E), ("aux_loss_bwd", bwd_not_centred),
                      ("gate_shares", shares_unnormalised)):
        with monkeypatch.context() as m:
            m.setattr(orc, name, bad)
            with pytest.raises(AssertionError):
                _aux_pins()
    _aux_pins()


# ------------------------------------------------------------ two-matrix GELU expert (Eq. 1 as printed)
def _gelu_pins():
    # closed forms: gelu(z) = z Phi(z); Phi(1) = 0.8413447460685429 (standard normal table value)
    z = np.array([0.0, 1.0, -1.0, 8.0])
    np.testing.assert_allclose(orc.gelu(z), [0.0, 0.8413447460685429, -0.15865525393145707, 8.0], rtol=1e-14, atol=1e-14)
    # a 1x1 "expert": y = gelu(x a) b;  dy/dx at z = 0 is a b / 2, at z = 1 it is a b (Phi(1) + phi(1))
    for zz, slope in ((0.0, 0.5), (1.0, 0.8413447460685429 + 0.24197072451914337)):
        x, a, b = np.array([[1.0]]), np.array([[zz]]), np.array([[3.0]])
        zv, h, y = orc.gelu_ffn(x, a, b)
        dx, dWa, dWb, dz = orc.gelu_ffn_bwd(x, a, b, zv, np.array([[1.0]]))
        np.testing.assert_allclose(dz, [[3.0 * slope]], rtol=1e-14)
        np.testing.assert_allclose(dx, [[3.0 * slope * zz]], rtol=1e-14, atol=1e-15)
        np.testing.assert_allclose(dWa, [[3.0 * slope]], rtol=1e-14)
        np.testing.assert_allclose(dWb, h, rtol=1e-14)
    # the whole layer with two matrices per expert against a dense masked evaluation in torch
    for cfg in (small_cfg(T=24, d=8, E=6, k=2, d_ff=12, ffn="gelu"),
                small_cfg(T=16, d=8, E=5, k=3, d_ff=6, ffn="gelu", gate="sigmoid", n_shared=2, d_ff_shared=7)):
        p = problem(cfg)
        assert "Wu" not in p and "Wsu" not in p
        o = oracle_inputs(p)
        out = orc.layer_fwd_bwd(o["logits"], o["X"], o["dY"], o["Wg"], None, o["Wd"], cfg.k, cfg.gate, cfg.renorm,
                                o.get("Wsg"), None, o.get("Wsd"), want_dlogits=True)
        tX = torch.tensor(o["X"], requires_grad=True)
        tWa = torch.tensor(o["Wg"], requires_grad=True)
        tWb = torch.tensor(o["Wd"], requires_grad=True)
        tw = torch.tensor(out["topk_w"], requires_grad=True)
        wfull = torch.zeros(cfg.T, cfg.E, dtype=torch.float64).scatter(1, torch.tensor(out["topk_idx"].astype(np.int64)), tw)
        Y = torch.zeros(cfg.T, cfg.d, dtype=torch.float64)
        for e in range(cfg.E):
            Y = Y + wfull[:, e:e + 1] * (torch.nn.functional.gelu(tX @ tWa[e]) @ tWb[e])
        shared = {}
        if cfg.n_shared:
            shared = {n: torch.tensor(o[n], requires_grad=True) for n in ("Wsg", "Wsd")}
            for s_ in range(cfg.n_shared):
                Y = Y + torch.nn.functional.gelu(tX @ shared["Wsg"][s_]) @ shared["Wsd"][s_]
        (Y * torch.tensor(o["dY"])).sum().backward()
        tol = dict(rtol=1e-10, atol=1e-12)
        np.testing.assert_allclose(out["Y"], Y.detach().numpy(), **tol)
        np.testing.assert_allclose(out["dX"], tX.grad.numpy(), **tol)
        np.testing.assert_allclose(out["dWg"], tWa.grad.numpy(), **tol)
        np.testing.assert_allclose(out["dWd"], tWb.grad.numpy(), **tol)
        np.testing.assert_allclose(out["dw"], tw.grad.numpy(), **tol)
        assert not out["dWu"].any() and not out["U"].any()
        if cfg.n_shared:
            np.testing.assert_allclose(out["dWsg"], shared["Wsg"].grad.numpy(), **tol)
            np.testing.assert_allclose(out["dWsd"], shared["Wsd"].grad.numpy(), **tol)
    # one expert, top-1: two plain matrix products around the activation
    cfg = small_cfg(T=10, d=6, E=1, k=1, d_ff=9, ffn="gelu")
    o = oracle_inputs(problem(cfg))
    out = orc.layer_fwd_bwd(o["logits"], o["X"], o["dY"], o["Wg"], None, o["Wd"], 1)
    np.testing.assert_allclose(out["Y"], orc.gelu(o["X"] @ o["Wg"][0]) @ o["Wd"][0], rtol=1e-12, atol=1e-14)


def test_two_matrix_gelu_ffn():
    _gelu_pins()


def test_planted_mistakes_in_gelu_ffn_are_caught(monkeypatch):
    real_bwd, real_gelu = orc.gelu_ffn_bwd, orc.gelu

    def bwd_without_density_term(x, Wa, Wb, z, dy):      # f'(z) = Phi(z) only
        from scipy.special import erf
        dz = (dy @ Wb.T) * 0.5 * (1.0 + erf(z / np.sqrt(2.0)))
        return dz @ Wa.T, x.T @ dz, real_gelu(z).T @ dy, dz

    def tanh_gelu(z):                                     # the tanh approximation instead of z Phi(z)
        return 0.5 * z * (1.0 + np.tanh(np.sqrt(2.0 / np.pi) * (z + 0.044715 * z ** 3)))

    def bwd_swapped(x, Wa, Wb, z, dy):                    # dWb from the pre-activation instead of the activation
        dx, dWa, _, dz = real_bwd(x, Wa, Wb, z, dy)
        return dx, dWa, z.T @ dy, dz

    for name, bad in (("gelu_ffn_bwd", bwd_without_density_term), ("gelu", tanh_gelu), ("gelu_ffn_bwd", bwd_swapped)):
        with monkeypatch.context() as m:
            m.setattr(orc, name, bad)
            with pytest.raises(AssertionError):
                _gelu_pins()
    _gelu_pins()
