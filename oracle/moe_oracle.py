"""Plain CPU oracle of one GPU's share of an MoE layer's training step.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this module;
only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg call it.
It shares no code with the HIP path and never calls it.

What it computes is the MoE layer of Eq. 3 of the paper,
    MoE(x) = sum over i in argtopk(g(x)) of g(x)_i * f(x W_i^A) W_i^B,
with the expert body of Eq. 1 (FFN(x) = f(x W^A) W^B), evaluated exactly as the
definition says and then differentiated by hand.  The readings the paper leaves
open are taken as follows (each is a choice of this build, not of the paper):
  * f(x W^A) is SwiGLU: W^A is the pair (Wg, Wu), f(x W^A) = silu(x Wg) * (x Wu),
    silu(z) = z / (1 + exp(-z));  W^B is Wd.  For the paper's synthetic GPT-MoE models (a
    sparsified GPT-3: two matrices per expert, d_ffn = 4 d_model) Wu is None and f is GELU,
    gelu(z) = z Phi(z); the paper does not name f.
  * g is a softmax over all E logits, or an element-wise sigmoid; the k selected
    scores are divided by their sum when renorm is set.
  * selection is on the raw fp32 logits (both gates are increasing in the logit):
    descending logit, ties to the lower expert index; output slot j holds rank j.
  * no token is dropped and no capacity is applied (evaluation setup of the paper:
    every token-expert assignment is computed).
  * rows are grouped by expert with a stable counting sort over the flat
    assignment index a = t*k + j.
  * shared experts are always-on experts of weight 1, summed into the output
    (Eq. 2: experts summed along d_ff).
  * the gating network that produces the logits (router_fwd / router_bwd) is one
    linear map without bias; the paper only calls it "lightweight".
  * the auxiliary load-balancing loss (aux_loss / aux_loss_bwd) is the product form
    alpha * E * sum_e (load share of e) * (mean score share of e); the paper gives the
    weight and a citation, not the formula.
Every function works in the real type R (float64 unless told otherwise) on the
input values widened to R; no intermediate is rounded to a narrower type.

Parity pins (tests/test_oracle_pins.py): hand-worked closed forms stored under
tests/golden/, invariants, a dense all-experts-masked evaluation differentiated by
torch autograd, central finite differences, and special cases that reduce to plain
matrix products.  The paper prints no worked numeric example of this path, so no
pin comes from printed paper values.
"""
from __future__ import annotations

import numpy as np
from scipy.special import erf as _erf

DEFAULT_R = np.float64


# --------------------------------------------------------------------------- router
def router_fwd(X, Wr, R=DEFAULT_R):
    """Logits of the gating network g of Eq. 3, read as one linear map of the token:
    logits[t, e] = sum_c X[t, c] * Wr[c, e]   (X [T, d], Wr [d, E])."""
    return np.asarray(X).astype(R) @ np.asarray(Wr).astype(R)


def router_bwd(X, Wr, dlogits, R=DEFAULT_R):
    """Adjoint of router_fwd: dWr[c, e] = sum_t X[t, c] dlogits[t, e];  dX[t, c] = sum_e dlogits[t, e] Wr[c, e]."""
    X = np.asarray(X).astype(R)
    Wr = np.asarray(Wr).astype(R)
    dl = np.asarray(dlogits).astype(R)
    dWr = np.zeros_like(Wr)
    for t in range(X.shape[0]):
        dWr += np.outer(X[t], dl[t])
    return dl @ Wr.T, dWr


# --------------------------------------------------------------------------- gating
def gate_scores(logits, gate, R=DEFAULT_R):
    """g(x) of Eq. 3 from router logits [T, E]: softmax over experts, or sigmoid."""
    z = np.asarray(logits).astype(R)
    if gate == "softmax":
        z = z - z.max(axis=1, keepdims=True)
        e = np.exp(z)
        return e / e.sum(axis=1, keepdims=True)
    if gate == "sigmoid":
        return 1.0 / (1.0 + np.exp(-z))
    raise ValueError(f"unknown gate {gate!r}")


def select_topk(logits, k):
    """argtopk of Eq. 3 on the raw logits: descending value, ties to the lower index."""
    lg = np.asarray(logits)
    T, E = lg.shape
    if not 1 <= k <= E:
        raise ValueError("need 1 <= k <= E")
    idx = np.empty((T, k), dtype=np.int32)
    for t in range(T):
        row = lg[t]
        order = sorted(range(E), key=lambda e: (-float(row[e]), e))
        idx[t] = order[:k]
    return idx


def route(logits, k, gate="softmax", renorm=True, R=DEFAULT_R):
    """Top-k gating: indices [T, k] int32 and combine weights [T, k] (Eq. 3's g(x)_i)."""
    idx = select_topk(logits, k)
    s = gate_scores(logits, gate, R)
    w = np.take_along_axis(s, idx.astype(np.int64), axis=1)
    if renorm:
        w = w / w.sum(axis=1, keepdims=True)
    return idx, w


def route_bwd(logits, idx, dw, gate="softmax", renorm=True, R=DEFAULT_R):
    """Gradient of the combine weights with respect to the logits, selection held fixed."""
    s = gate_scores(logits, gate, R)
    T, E = s.shape
    ii = idx.astype(np.int64)
    ssel = np.take_along_axis(s, ii, axis=1)
    dw = np.asarray(dw).astype(R)
    if renorm:
        tot = ssel.sum(axis=1, keepdims=True)
        w = ssel / tot
        dssel = (dw - (dw * w).sum(axis=1, keepdims=True)) / tot
    else:
        dssel = dw
    ds = np.zeros((T, E), dtype=R)
    np.put_along_axis(ds, ii, dssel, axis=1)
    if gate == "softmax":
        return s * (ds - (s * ds).sum(axis=1, keepdims=True))
    return ds * s * (1.0 - s)


# ----------------------------------------------------------------- auxiliary loss
def gate_shares(logits, gate, R=DEFAULT_R):
    """The gate's scores as shares that sum to one over the E experts of a token:
    the softmax itself, or the sigmoid scores divided by their sum."""
    s = gate_scores(logits, gate, R)
    return s if gate == "softmax" else s / s.sum(axis=1, keepdims=True)


def aux_loss(logits, counts, k, alpha, gate="softmax", R=DEFAULT_R):
    """Auxiliary load-balancing loss.  The evaluation setup of the paper trains with one
    (weight 0.001, swept to 0.1 in its sensitivity study) and cites the GShard form without
    printing it; the reading taken here is the usual product form of that family,

        L = alpha * E * sum_e f_e * P_e,
        f_e = counts[e] / (T k)   share of the T*k assignments that expert e received,
        P_e = (1/T) sum_t p_te    mean share of expert e in the gate's scores,

    which equals alpha whenever either the loads or the scores are uniform.
    Returns (L, P[E])."""
    p = gate_shares(logits, gate, R)
    T, E = p.shape
    f = np.asarray(counts).astype(R) / R(T * k)
    P = p.sum(axis=0) / R(T)
    return R(alpha) * R(E) * (f * P).sum(), P


def aux_loss_bwd(logits, counts, k, alpha, gate="softmax", dloss=1.0, R=DEFAULT_R):
    """d(aux_loss)/d(logits) [T, E], loads f held constant (they are piecewise constant in
    the logits), times the upstream scalar dloss.
        c_e = dL/dp_te = alpha E f_e / T                     (the same for every token)
        softmax:  dz_te = p_te (c_e - sum_j p_tj c_j)
        sigmoid:  p = s / S, S = sum_j s_j:  ds_te = (c_e - sum_j p_tj c_j) / S,
                  dz_te = ds_te s_te (1 - s_te)"""
    p = gate_shares(logits, gate, R)
    T, E = p.shape
    c = R(dloss) * R(alpha) * R(E) * (np.asarray(counts).astype(R) / R(T * k)) / R(T)
    centred = c[None, :] - (p * c[None, :]).sum(axis=1, keepdims=True)
    if gate == "softmax":
        return p * centred
    s = gate_scores(logits, gate, R)
    return centred / s.sum(axis=1, keepdims=True) * s * (1.0 - s)


# ------------------------------------------------------------------------- dispatch
def dispatch_plan(idx, E):
    """Stable counting sort of the assignments a = t*k + j by expert.

    counts[e]  number of assignments of expert e (T[e, d] of the paper's token
               dispatching, with a single device);
    offsets    exclusive prefix sum, offsets[E] = T*k;
    row_of[a]  row of assignment a in the expert-contiguous order;
    src_of     inverse of row_of.
    """
    flat = np.asarray(idx).reshape(-1)
    A = flat.shape[0]
    counts = np.zeros(E, dtype=np.int32)
    for a in range(A):
        counts[flat[a]] += 1
    offsets = np.zeros(E + 1, dtype=np.int32)
    for e in range(E):
        offsets[e + 1] = offsets[e] + counts[e]
    nxt = offsets[:E].copy()
    row_of = np.empty(A, dtype=np.int32)
    src_of = np.empty(A, dtype=np.int32)
    for a in range(A):
        e = flat[a]
        r = nxt[e]
        nxt[e] += 1
        row_of[a] = r
        src_of[r] = a
    return counts, offsets, row_of, src_of


def permute_rows(X, row_of, k, R=DEFAULT_R):
    """Xp[row_of[t*k + j]] = X[t]."""
    X = np.asarray(X).astype(R)
    A = row_of.shape[0]
    Xp = np.empty((A, X.shape[1]), dtype=R)
    for a in range(A):
        Xp[row_of[a]] = X[a // k]
    return Xp


# ------------------------------------------------------------------------ expert FFN
def silu(z):
    return z / (1.0 + np.exp(-z))


def swiglu_ffn(x, Wg, Wu, Wd):
    """Eq. 1 with the SwiGLU reading: returns (g, u, h, y) for rows x."""
    g = x @ Wg
    u = x @ Wu
    h = silu(g) * u
    return g, u, h, h @ Wd


def swiglu_ffn_bwd(x, Wg, Wu, Wd, g, u, dy):
    """Chain rule on Eq. 1: returns (dx, dWg, dWu, dWd, dg, du)."""
    sig = 1.0 / (1.0 + np.exp(-g))
    h = g * sig * u
    dh = dy @ Wd.T
    du = dh * (g * sig)
    dg = dh * u * (sig * (1.0 + g * (1.0 - sig)))
    dx = dg @ Wg.T + du @ Wu.T
    return dx, x.T @ dg, x.T @ du, h.T @ dy, dg, du


def gelu(z):
    """x * Phi(x) with the standard normal distribution function Phi."""
    return 0.5 * z * (1.0 + _erf(z / np.sqrt(2.0)))


def gelu_ffn(x, Wa, Wb):
    """Eq. 1 as printed, FFN(x) = f(x W^A) W^B, with f = GELU: returns (z, h, y) for rows x."""
    z = x @ Wa
    h = gelu(z)
    return z, h, h @ Wb


def gelu_ffn_bwd(x, Wa, Wb, z, dy):
    """Chain rule on the two-matrix FFN: returns (dx, dWa, dWb, dz);
    f'(z) = Phi(z) + z phi(z), phi the standard normal density."""
    dh = dy @ Wb.T
    dz = dh * (0.5 * (1.0 + _erf(z / np.sqrt(2.0))) + z * np.exp(-0.5 * z * z) / np.sqrt(2.0 * np.pi))
    return dz @ Wa.T, x.T @ dz, gelu(z).T @ dy, dz


def ffn(x, Wg, Wu, Wd):
    """The expert body: SwiGLU with three matrices, or (Wu is None) the two-matrix GELU FFN
    with W^A = Wg, W^B = Wd.  Returns (g, u, h, y); in the two-matrix case g is the
    pre-activation and u is zero."""
    if Wu is None:
        z, h, y = gelu_ffn(x, Wg, Wd)
        return z, np.zeros_like(z), h, y
    return swiglu_ffn(x, Wg, Wu, Wd)


def ffn_bwd(x, Wg, Wu, Wd, g, u, dy):
    """Returns (dx, dWg, dWu, dWd, dg, du); dWu and du are zero in the two-matrix case."""
    if Wu is None:
        dx, dWa, dWb, dz = gelu_ffn_bwd(x, Wg, Wd, g, dy)
        return dx, dWa, np.zeros_like(dWa), dWb, dz, np.zeros_like(dz)
    return swiglu_ffn_bwd(x, Wg, Wu, Wd, g, u, dy)


def _mat(W, i, R):
    return None if W is None else np.asarray(W[i]).astype(R)


def expert_fwd(Xp, offsets, Wg, Wu, Wd, R=DEFAULT_R):
    """Every expert on its own contiguous block of rows; experts without rows do nothing."""
    Xp = np.asarray(Xp).astype(R)
    n, d = Xp.shape
    E = len(offsets) - 1
    F = np.asarray(Wg[0]).shape[1]
    G = np.zeros((n, F), dtype=R)
    U = np.zeros((n, F), dtype=R)
    H = np.zeros((n, F), dtype=R)
    Yp = np.zeros((n, d), dtype=R)
    for e in range(E):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        if hi == lo:
            continue
        g, u, h, y = ffn(Xp[lo:hi], _mat(Wg, e, R), _mat(Wu, e, R), _mat(Wd, e, R))
        G[lo:hi], U[lo:hi], H[lo:hi], Yp[lo:hi] = g, u, h, y
    return G, U, H, Yp


def expert_bwd(Xp, offsets, Wg, Wu, Wd, G, U, dYp, R=DEFAULT_R):
    """dX rows and dense per-expert weight gradients (zero for experts without rows)."""
    Xp = np.asarray(Xp).astype(R)
    dYp = np.asarray(dYp).astype(R)
    n, d = Xp.shape
    E = len(offsets) - 1
    F = np.asarray(Wg[0]).shape[1]
    dXp = np.zeros((n, d), dtype=R)
    dWg = np.zeros((E, d, F), dtype=R)
    dWu = np.zeros((E, d, F), dtype=R)
    dWd = np.zeros((E, F, d), dtype=R)
    dG = np.zeros((n, F), dtype=R)
    dU = np.zeros((n, F), dtype=R)
    for e in range(E):
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        if hi == lo:
            continue
        out = ffn_bwd(Xp[lo:hi], _mat(Wg, e, R), _mat(Wu, e, R), _mat(Wd, e, R), np.asarray(G[lo:hi]).astype(R),
                      np.asarray(U[lo:hi]).astype(R), dYp[lo:hi])
        dXp[lo:hi], dWg[e], dWu[e], dWd[e], dG[lo:hi], dU[lo:hi] = out
    return dXp, dWg, dWu, dWd, dG, dU


def shared_fwd(X, Wsg, Wsu, Wsd, R=DEFAULT_R):
    """Always-on experts on all rows, outputs summed.  Returns (Gs [S,T,Fs], Us, Ysh [T,d])."""
    X = np.asarray(X).astype(R)
    S = len(Wsg)
    Gs, Us = [], []
    Ysh = np.zeros_like(X)
    for s in range(S):
        g, u, _, y = ffn(X, _mat(Wsg, s, R), _mat(Wsu, s, R), _mat(Wsd, s, R))
        Gs.append(g)
        Us.append(u)
        Ysh += y
    return np.stack(Gs), np.stack(Us), Ysh


def shared_bwd(X, Wsg, Wsu, Wsd, Gs, Us, dY, R=DEFAULT_R):
    """Returns (dXsh [T,d], dWsg, dWsu, dWsd) for the always-on experts."""
    X = np.asarray(X).astype(R)
    dY = np.asarray(dY).astype(R)
    S = len(Wsg)
    dX = np.zeros_like(X)
    dWsg, dWsu, dWsd = [], [], []
    for s in range(S):
        dx, a, b, c, _, _ = ffn_bwd(X, _mat(Wsg, s, R), _mat(Wsu, s, R), _mat(Wsd, s, R), np.asarray(Gs[s]).astype(R),
                                    np.asarray(Us[s]).astype(R), dY)
        dX += dx
        dWsg.append(a)
        dWsu.append(b)
        dWsd.append(c)
    return dX, np.stack(dWsg), np.stack(dWsu), np.stack(dWsd)


# --------------------------------------------------------------------------- combine
def combine(Yp, row_of, w, Yadd=None, R=DEFAULT_R):
    """The weighted sum of Eq. 3: Y[t] = Yadd[t] + sum_j w[t,j] * Yp[row_of[t*k+j]]."""
    Yp = np.asarray(Yp).astype(R)
    w = np.asarray(w).astype(R)
    T, k = w.shape
    d = Yp.shape[1]
    Y = np.zeros((T, d), dtype=R) if Yadd is None else np.asarray(Yadd).astype(R).copy()
    for t in range(T):
        for j in range(k):
            Y[t] += w[t, j] * Yp[row_of[t * k + j]]
    return Y


def unpermute(dXp, row_of, k, dXadd=None, R=DEFAULT_R):
    """dX[t] = dXadd[t] + sum_j dXp[row_of[t*k+j]]  (adjoint of permute_rows)."""
    A = np.asarray(dXp).shape[0]
    ones = np.ones((A // k, k), dtype=R)
    return combine(dXp, row_of, ones, dXadd, R)


def combine_bwd(dY, Yp, row_of, w, R=DEFAULT_R):
    """dYp[row_of[a]] = w[a] * dY[t];  dw[t,j] = <dY[t], Yp[row_of[a]]>,  a = t*k+j."""
    dY = np.asarray(dY).astype(R)
    Yp = np.asarray(Yp).astype(R)
    w = np.asarray(w).astype(R)
    T, k = w.shape
    dYp = np.empty_like(Yp)
    dw = np.empty((T, k), dtype=R)
    for t in range(T):
        for j in range(k):
            r = row_of[t * k + j]
            dYp[r] = w[t, j] * dY[t]
            dw[t, j] = np.dot(dY[t], Yp[r])
    return dYp, dw


# ------------------------------------------------------------------------ compaction
def active_experts(counts):
    """Ascending ids of experts that received at least one row, padded with -1, and their number."""
    counts = np.asarray(counts)
    ids = [e for e in range(counts.shape[0]) if counts[e] > 0]
    out = np.full(counts.shape[0], -1, dtype=np.int32)
    out[:len(ids)] = ids
    return out, np.int32(len(ids))


def compact(dense, active_ids, n_active):
    """Slot i of the compact gradient buffer holds expert active_ids[i]."""
    return np.stack([dense[int(active_ids[i])] for i in range(int(n_active))]) if n_active else dense[:0]


# ---------------------------------------------------------------------- whole layer
def layer_fwd_bwd(logits, X, dY, Wg, Wu, Wd, k, gate="softmax", renorm=True,
                  Wsg=None, Wsu=None, Wsd=None, R=DEFAULT_R, want_dlogits=False, aux_alpha=0.0):
    """One forward and backward pass of the layer; returns every intermediate by name.
    With aux_alpha > 0 the auxiliary load-balancing loss is evaluated too and its gradient
    (upstream gradient 1) is part of dlogits."""
    E = len(Wg)
    X = np.asarray(X).astype(R)
    dY = np.asarray(dY).astype(R)
    o = {}
    o["topk_idx"], o["topk_w"] = route(logits, k, gate, renorm, R)
    o["counts"], o["offsets"], o["row_of"], o["src_of"] = dispatch_plan(o["topk_idx"], E)
    o["Xp"] = permute_rows(X, o["row_of"], k, R)
    o["G"], o["U"], o["H"], o["Yp"] = expert_fwd(o["Xp"], o["offsets"], Wg, Wu, Wd, R)
    shared = Wsg is not None and len(Wsg) > 0
    if shared:
        o["Gs"], o["Us"], o["Ysh"] = shared_fwd(X, Wsg, Wsu, Wsd, R)
    o["Y"] = combine(o["Yp"], o["row_of"], o["topk_w"], o.get("Ysh"), R)
    if aux_alpha > 0:
        o["aux_loss"], o["aux_P"] = aux_loss(logits, o["counts"], k, aux_alpha, gate, R)
    # backward
    o["dYp"], o["dw"] = combine_bwd(dY, o["Yp"], o["row_of"], o["topk_w"], R)
    (o["dXp"], o["dWg"], o["dWu"], o["dWd"], o["dG"], o["dU"]) = expert_bwd(
        o["Xp"], o["offsets"], Wg, Wu, Wd, o["G"], o["U"], o["dYp"], R)
    o["active_ids"], o["n_active"] = active_experts(o["counts"])
    if shared:
        o["dXsh"], o["dWsg"], o["dWsu"], o["dWsd"] = shared_bwd(X, Wsg, Wsu, Wsd, o["Gs"], o["Us"], dY, R)
    o["dX"] = unpermute(o["dXp"], o["row_of"], k, o.get("dXsh"), R)
    if want_dlogits:
        o["dlogits"] = route_bwd(logits, o["topk_idx"], o["dw"], gate, renorm, R)
        if aux_alpha > 0:
            o["dlogits"] = o["dlogits"] + aux_loss_bwd(logits, o["counts"], k, aux_alpha, gate, 1.0, R)
    return o


def token_fwd_bwd(x, idx_t, w_t, dy, Wg, Wu, Wd, Wsg=None, Wsu=None, Wsd=None, R=DEFAULT_R):
    """Eq. 3 and its input gradient for ONE token given its selected experts and weights.

    Used to check sampled rows of Y, dX and dw at sizes where the whole layer is too
    slow on the CPU.  Returns (y [d], dx [d], dw [k]).
    """
    x = np.asarray(x).astype(R)[None, :]
    dy = np.asarray(dy).astype(R)[None, :]
    y = np.zeros_like(x)
    dx = np.zeros_like(x)
    dw = np.zeros(len(idx_t), dtype=R)
    for j, e in enumerate(idx_t):
        We = [_mat(W, int(e), R) for W in (Wg, Wu, Wd)]
        g, u, _, yj = ffn(x, *We)
        y += R(w_t[j]) * yj
        dw[j] = float((dy * yj).sum())
        dx += ffn_bwd(x, *We, g, u, R(w_t[j]) * dy)[0]
    if Wsg is not None:
        for s in range(len(Wsg)):
            We = [_mat(W, s, R) for W in (Wsg, Wsu, Wsd)]
            g, u, _, ys = ffn(x, *We)
            y += ys
            dx += ffn_bwd(x, *We, g, u, dy)[0]
    return y[0], dx[0], dw
