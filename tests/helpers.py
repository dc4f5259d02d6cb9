"""Shared test helpers: small seeded problems, error norms, golden-file parsing."""
from __future__ import annotations

import math
import os

import numpy as np
import torch

import workloads as wl

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def small_cfg(name="t", T=24, d=8, E=6, k=2, d_ff=12, n_shared=0, d_ff_shared=0, dtype="f32",
              gate="softmax", renorm=True, zipf_s=1.0, seed=0, routing="zipf", aux_alpha=0.0, ffn="swiglu"):
    return wl.MoEConfig(name, T=T, d=d, E=E, k=k, d_ff=d_ff, n_shared=n_shared, d_ff_shared=d_ff_shared,
                        dtype=dtype, gate=gate, renorm=renorm, zipf_s=zipf_s, seed=seed, routing=routing,
                        aux_alpha=aux_alpha, ffn=ffn)


def np64(t):
    """A torch tensor (any float dtype) or array as float64 numpy."""
    if isinstance(t, torch.Tensor):
        return t.detach().to("cpu", torch.float64).numpy()
    return np.asarray(t, dtype=np.float64)


def problem(cfg, unit_scale=True, device="cpu"):
    """Seeded inputs for cfg as a dict of torch tensors (weights on `device`)."""
    if unit_scale:
        xs, ws = wl.unit_scale_stds(cfg)
        gs = 1.0
    else:
        xs, ws, gs = wl.TOKEN_STD, wl.WEIGHT_STD, wl.GRAD_STD
    p = {"logits": wl.make_logits(cfg), "X": wl.make_tokens(cfg, xs), "dY": wl.make_grad_out(cfg, gs)}
    p.update(wl.make_weights(cfg, device, ws))
    return p


def oracle_inputs(p):
    """float64 numpy copies of a problem dict (the logits stay fp32: selection is on raw fp32)."""
    out = {}
    for key, v in p.items():
        out[key] = v.detach().cpu().numpy() if key == "logits" else np64(v)
    return out


def scale_rel_err(got, ref):
    """max |got - ref| / max |ref|  (the tolerance norm used for floating-point parity)."""
    got, ref = np64(got), np64(ref)
    den = float(np.abs(ref).max())
    if den == 0.0:
        return float(np.abs(got).max())
    return float(np.abs(got - ref).max()) / den


def _eval(expr, env):
    return float(eval(expr, {"__builtins__": {}}, env))


def read_route_golden():
    cases = []
    with open(os.path.join(GOLDEN, "route_closed_forms.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            head, lg, idx, w = [s.strip() for s in line.split("|")]
            gate, renorm, k = head.split()
            logits = []
            for tok in lg.split():
                logits.append(-1.0e4 if tok == "m" else math.log(float(tok[2:])))
            weights = [float(a) / float(b) for a, b in (x.split("/") for x in w.split())]
            cases.append((gate, bool(int(renorm)), int(k), logits, [int(i) for i in idx.split()], weights))
    return cases


def read_swiglu_golden():
    env = {"L": math.log(3.0)}
    out = {}
    with open(os.path.join(GOLDEN, "swiglu_closed_form.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            name, rhs = [s.strip() for s in line.split("=", 1)]
            rows = [[_eval(tok, env) for tok in row.split()] for row in rhs.split(";")]
            out[name] = np.array(rows, dtype=np.float64)
    return out
