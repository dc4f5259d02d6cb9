#!/usr/bin/env python3
"""Benchmark of the MoE-layer hot path on one MI355X.

One "step" is one forward+backward pass of the whole path (route, dispatch, routed and shared
expert grouped GEMMs, combine; combine-bwd, dH/dX/dW grouped GEMMs with compacted dW, un-permute, gate backward)
over one batch of seeded synthetic input that is already resident in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config dsv3|qwen|phi|stress|tiny]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import workloads as wl  # noqa: E402

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
MFMA_BF16_PEAK_TF = 2500.0   # dense bf16 matrix peak, published
FP32_VEC_PEAK_TF = 157.3

GEMM_LABELS = ("gemm_fwd_gate_up", "gemm_fwd_down", "gemm_bwd_dh", "gemm_bwd_dx", "gemm_bwd_dwd", "gemm_bwd_dwgu",
               "gemm_bwd_dw_light")
LIGHT_GROUP_ROWS = 256       # routed experts with at most this many rows take the light weight-gradient kernels
PROBE_BYTES = 1 << 30        # size of the calibration copy
PROBE_LAUNCHES = 5
COLD_STEPS = 3               # steps of the cold-cache variant
# kernel behind each profiling label on the bf16 LDS-DMA path, as rocprofv3 names it (one label = one kernel symbol)
SYMBOL = {
    "gemm_fwd_gate_up": "moe::row_gemm_kernel<moe::RowCores<2, 2, false>, 2, 1, false>(moe::RowGemm)",
    "gemm_fwd_down": "moe::row_gemm_kernel<moe::RowCores<2, 1, false>, 1, 0, false>(moe::RowGemm)",
    "gemm_bwd_dh": "moe::row_gemm_kernel<moe::RowCores<2, 1, true>, 1, 2, true>(moe::RowGemm)",
    "gemm_bwd_dx": "moe::row_gemm_kernel<moe::RowCores<2, 1, true>, 1, 0, true>(moe::RowGemm)",
    "gemm_bwd_dwd": "moe::w_gemm_kernel<moe::MfmaDmaCore<256, 256, 1, false, false, 2, 2, 1>, 1>(moe::WGemm)",
    "gemm_bwd_dwgu": "moe::w_gemm_kernel<moe::MfmaDmaCore<256, 128, 2, false, false, 2, 2, 1>, 2>(moe::WGemm)",
    "gemm_bwd_dw_light": "moe::w_gemm_kernel<moe::MfmaDmaCore<128, 128, 1, false, false, 2, 2, 0>, 1>(moe::WGemm)",
}


def algorithmic_work(cfg: wl.MoEConfig, counts):
    """Per step: FLOPs of each GEMM label over real rows only, bytes of each streaming kernel."""
    b = 4 if cfg.dtype == "f32" else 2
    A, T, d, F, k = cfg.A, cfg.T, cfg.d, cfg.d_ff, cfg.k
    routed = A * d * F
    shared = cfg.n_shared * T * d * cfg.d_ff_shared
    unit = routed + shared
    m_in = 2.0 if cfg.ffn == "swiglu" else 1.0   # matrices on the input side of the expert (Wg, Wu | W^A)
    flops = {"gemm_fwd_gate_up": 2.0 * m_in * unit, "gemm_fwd_down": 2.0 * unit, "gemm_bwd_dh": 2.0 * unit,
             "gemm_bwd_dx": 2.0 * m_in * unit, "gemm_bwd_dwd": 2.0 * unit, "gemm_bwd_dwgu": 2.0 * m_in * unit}
    if cfg.dtype == "bf16" and d % 64 == 0 and F % 64 == 0:
        light = int(counts[counts <= LIGHT_GROUP_ROWS].sum()) * d * F
        flops["gemm_bwd_dw_light"] = (2.0 + 2.0 * m_in) * light  # two launches: dWd, then dWg (and dWu)
        flops["gemm_bwd_dwd"] -= 2.0 * light
        flops["gemm_bwd_dwgu"] -= 2.0 * m_in * light
    has_sh = 1 if cfg.n_shared else 0
    byts = {
        "route_kernel": T * cfg.E * 4 + T * k * 8,
        "route_bwd_kernel": 2 * T * cfg.E * 4 + T * k * 8,
        "dispatch_rows": (1 + k) * T * d * b + A * 4,
        # two launches per step: Y (weights, + shared output) and dX (unit weights, + shared dX)
        "combine_kernel": 2 * ((k + 1 + has_sh) * T * d * b + A * 4) + A * 4,
        "combine_bwd_kernel": (1 + 2 * k) * T * d * b + A * 12,
    }
    return flops, byts


def measured_traffic(cfg_name, symbol):
    """HBM bytes per launch of `symbol` from the committed counter summary of this workload, or None."""
    from paper_2502_02581_amd.rocprof_summary import read_traffic

    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{cfg_name}.txt")
    if not os.path.exists(path):
        return None
    return read_traffic(path).get(symbol)


class LazyExperts:
    """Expert weights that stay on the GPU; the oracle receives one expert at a time as fp32 numpy."""

    def __init__(self, w: torch.Tensor):
        self.w = w

    def __len__(self):
        return self.w.shape[0]

    def __getitem__(self, e):
        return self.w[int(e)].float().cpu().numpy()


def cpu_baseline(cfg, inp, weights, budget_tokens):
    """Times the oracle, as it stands, on the first `budget_tokens` tokens of the same workload."""
    from oracle import moe_oracle as orc

    n = min(budget_tokens, cfg.T)
    lg = inp["logits"][:n].numpy()
    X = inp["X"][:n].float().numpy()
    dY = inp["dY"][:n].float().numpy()
    W = {k: LazyExperts(v) for k, v in weights.items()}
    t0 = time.perf_counter()
    orc.layer_fwd_bwd(lg, X, dY, W["Wg"], W.get("Wu"), W["Wd"], cfg.k, cfg.gate, cfg.renorm,
                      W.get("Wsg"), W.get("Wsu"), W.get("Wsd"))
    dt = time.perf_counter() - t0
    return {"value": n / dt, "unit": "tokens/s", "cores": torch.get_num_threads(), "kind": "oracle",
            "sample": f"first {n} of {cfg.T} tokens of the same workload, fwd+bwd, fp64 numpy oracle, {dt:.1f} s"}


def verify(cfg, inp, weights, hp):
    """Sampled check of the timed path against the oracle; a wrong result must never be timed."""
    import numpy as np
    from oracle import moe_oracle as orc

    W = {k: LazyExperts(v) for k, v in weights.items()}
    idx = hp.b["topk_idx"].cpu().numpy()
    w = hp.b["topk_w"].cpu().numpy().astype(np.float64)
    worst = 0.0
    for t in (0, cfg.T // 2, cfg.T - 1):
        y, dx, _ = orc.token_fwd_bwd(inp["X"][t].double().numpy(), idx[t], w[t], inp["dY"][t].double().numpy(),
                                     W["Wg"], W.get("Wu"), W["Wd"], W.get("Wsg"), W.get("Wsu"), W.get("Wsd"))
        for got, ref in ((hp.b["Y"][t], y), (hp.b["dX"][t], dx)):
            err = float(np.abs(got.double().cpu().numpy() - ref).max() / np.abs(ref).max())
            worst = max(worst, err)
    tol = 1e-4 if cfg.dtype == "f32" else 2e-2
    if not worst <= tol:
        raise SystemExit(f"bench.py: the hot path disagrees with the oracle on sampled tokens (error {worst:.3e} > {tol})")
    return worst


CPU_SAMPLE_TOKENS = {"tiny": 256, "qwen": 1024, "phi": 256, "dsv3": 64, "stress": 1024, "gpt-s": 2048, "gpt-l": 512}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="dsv3", choices=list(wl.CONFIGS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--overlap-shared", action="store_true",
                    help="run the shared experts on a second stream (per-kernel durations then overlap)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is the one-GPU hot path; it has no multi-GPU mode (run with --gpus 1)",
              file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)

    import paper_2502_02581_amd as moe

    cfg = wl.CONFIGS[args.config]
    dev = "cuda:0"
    torch.cuda.set_device(0)
    inp = {"logits": wl.make_logits(cfg), "X": wl.make_tokens(cfg), "dY": wl.make_grad_out(cfg)}
    weights = wl.make_weights(cfg, dev)
    g = {k: v.to(dev) for k, v in inp.items()}
    shape = moe.MoEShape(cfg.T, cfg.d, cfg.E, cfg.k, cfg.d_ff, cfg.dtype, cfg.gate, cfg.renorm)
    hp = moe.MoEHotPath(shape, cfg.n_shared, cfg.d_ff_shared, dev, overlap_shared=args.overlap_shared,
                        aux_alpha=cfg.aux_alpha)
    sh = [weights.get("Wsg"), weights.get("Wsu"), weights.get("Wsd")]

    def step():
        hp.forward(g["logits"], g["X"], weights["Wg"], weights.get("Wu"), weights["Wd"], *sh)
        hp.backward(g["dY"], g["X"], weights["Wg"], weights.get("Wu"), weights["Wd"], *sh)

    for _ in range(max(1, args.warmup)):
        step()
    torch.cuda.synchronize()
    sampled_err = verify(cfg, inp, weights, hp)
    moe.moe_profile_enable(True)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0

    # one calibration copy of known size (outside the timed region): a profiler's HBM counters are scaled by it
    probe = torch.empty(2, PROBE_BYTES, dtype=torch.uint8, device=dev)
    probe.fill_(1)   # touches both halves, so that the copy is not timed on fresh pages
    for _ in range(PROBE_LAUNCHES):
        moe.moe_copy_probe(probe[0], probe[1])
    torch.cuda.synchronize()
    prof = moe.moe_profile_report()
    moe.moe_profile_enable(False)
    # cold-cache variant (outside the timed region, reported beside `value`): L2 and the infinity cache are
    # overwritten before every step by filling the 2 GiB probe buffer, and each step is timed on its own
    cold = []
    for _ in range(COLD_STEPS):
        probe.fill_(2)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        step()
        torch.cuda.synchronize()
        cold.append(time.perf_counter() - t1)
    del probe
    probe_ms = prof.pop("copy_probe_kernel")[1] / PROBE_LAUNCHES

    ms_per_step = dt / args.steps * 1e3
    counts = hp.b["counts"].cpu()
    flops, byts = algorithmic_work(cfg, counts)
    kernels = {}
    for label, (n, ms) in prof.items():
        per_step_ms = ms / args.steps
        ent = {"launches_per_step": n / args.steps, "ms_per_step": round(per_step_ms, 4)}
        if label in flops and per_step_ms > 0:
            ent["tflops"] = round(flops[label] / (per_step_ms * 1e-3) / 1e12, 2)
            ent["frac_mfma_peak"] = round(ent["tflops"] / (MFMA_BF16_PEAK_TF if cfg.dtype == "bf16" else FP32_VEC_PEAK_TF), 4)
        if label in byts and per_step_ms > 0:
            ent["gbs"] = round(byts[label] / (per_step_ms * 1e-3) / 1e9, 1)
            ent["frac_hbm_peak"] = round(ent["gbs"] / HBM_PEAK_GBS, 4)
        kernels[label] = ent
    gemm_ms = sum(kernels[l]["ms_per_step"] for l in GEMM_LABELS if l in kernels)
    gemm_tflops = sum(flops.values()) / (gemm_ms * 1e-3) / 1e12 if gemm_ms > 0 else 0.0
    dom = max((l for l in GEMM_LABELS if l in kernels), key=lambda l: kernels[l]["ms_per_step"])
    dom_n, dom_ms = prof[dom]
    peak = MFMA_BF16_PEAK_TF if cfg.dtype == "bf16" else FP32_VEC_PEAK_TF
    achieved = flops[dom] * args.steps / (dom_ms * 1e-3) / 1e12
    dma_path = cfg.dtype == "bf16" and cfg.d % 64 == 0 and cfg.d_ff % 64 == 0   # SYMBOL names that path's kernels
    roofline = {"bound": "mfma" if cfg.dtype == "bf16" else "alu", "kernel": dom, "symbol": SYMBOL[dom] if dma_path else None,
                "achieved": round(achieved, 2), "peak": peak, "unit": "TFLOP/s", "frac": round(achieved / peak, 4),
                "avg_launch_ms": round(dom_ms / dom_n, 4), "launches": dom_n,
                "flop_per_launch_avg": flops[dom] * args.steps / dom_n,
                "traffic": measured_traffic(cfg.name, SYMBOL[dom]) if dma_path else None}

    out = {
        "metric": "moe_layer_fwd_bwd_tokens_per_s", "value": round(cfg.T / (ms_per_step * 1e-3), 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: T={cfg.T} d={cfg.d} E={cfg.E} top-{cfg.k} {cfg.gate} d_ff={cfg.d_ff} "
                               f"shared={cfg.n_shared}x{cfg.d_ff_shared} routing={cfg.routing}(s={cfg.zipf_s}) seed={cfg.seed}",
                   "active_experts": int((counts > 0).sum()), "max_rows": int(counts.max()),
                   "load_share_std": round(float((counts.double() / counts.sum()).std(unbiased=False)), 5)},
        "grouped_gemm_tflops": round(gemm_tflops, 2), "grouped_gemm_frac_mfma_peak": round(gemm_tflops / peak, 4),
        "total_tflops": round(cfg.flops()["total"] / (ms_per_step * 1e-3) / 1e12, 2),
        "cold_cache_ms_per_step": round(sum(cold) / len(cold) * 1e3, 4),
        "roofline": roofline, "kernels": kernels,
        "copy_probe": {"bytes_each_way": PROBE_BYTES, "ms": round(probe_ms, 4),
                       "gbs": round(2 * PROBE_BYTES / (probe_ms * 1e-3) / 1e9, 1)}, "sampled_error_vs_oracle": float(f"{sampled_err:.3e}"),
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, inp, weights, CPU_SAMPLE_TOKENS[cfg.name])
    print(json.dumps(out))


if __name__ == "__main__":
    main()
