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
MFMA_PROBE_BLOCKS = 2048     # blocks (8 per CU) and rounds of the register-resident matrix loop
MFMA_PROBE_ITERS = 1000
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
    """(HBM bytes per launch of `symbol`, where that figure comes from).  The counters cannot be read
    from inside this process: the figure is the one `rocprofv3 --pmc` measured for this workload when the
    summary under profiles/ was last regenerated (the file names its command and the commit it ran)."""
    from paper_2502_02581_amd.rocprof_summary import read_traffic

    rel = os.path.join("profiles", f"hbm_traffic_{cfg_name}.txt")
    path = os.path.join(ROOT, rel)
    if not os.path.exists(path):
        return None, None
    commit = next((ln.split(":", 1)[1].strip() for ln in open(path) if ln.startswith("# commit:")), "not recorded")
    return read_traffic(path).get(symbol), f"{rel} (rocprofv3 --pmc FETCH_SIZE, WRITE_SIZE; kernels of commit {commit})"


class LazyExperts:
    """Expert weights that stay on the GPU; the oracle receives one expert at a time as fp32 numpy."""

    def __init__(self, w: torch.Tensor):
        self.w = w

    def __len__(self):
        return self.w.shape[0]

    def __getitem__(self, e):
        return self.w[int(e)].float().cpu().numpy()


def blas_threads():
    """Threads the BLAS behind numpy actually uses in this process."""
    try:
        from threadpoolctl import threadpool_info

        n = [int(i.get("num_threads", 0)) for i in threadpool_info() if i.get("user_api") == "blas"]
        if n:
            return max(n)
    except Exception:  # noqa: BLE001
        pass
    return os.cpu_count() or 1


def cpu_baseline(cfg, inp, weights, budget_s=15.0):
    """Times the oracle, as it stands, on a bounded sample of the same workload and scales it to the whole.

    Route and the dispatch plan run in full (they are cheap).  The expert work, which is all of the
    FLOPs, runs on whole experts of a deterministic subset -- the smallest and the median activated
    expert, the first shared expert, the largest expert, then further experts in descending size for
    as long as a short calibration product says they fit the budget (the largest and the shared one
    are cut to their leading rows if even they do not fit) -- so the sample's cost per FLOP is the
    full workload's by construction.  The operands are widened to fp64 outside the timed region: this is a
    compute rate, not a transfer rate."""
    import numpy as np
    from oracle import moe_oracle as orc

    R = np.float64
    lg = inp["logits"].numpy()
    t0 = time.perf_counter()
    idx, w = orc.route(lg, cfg.k, cfg.gate, cfg.renorm)
    counts, offsets, row_of, src_of = orc.dispatch_plan(idx, cfg.E)
    dt_plan = time.perf_counter() - t0
    # calibration: one fp64 product, sized to take well under a second
    a = np.ones((512, cfg.d), dtype=R)
    b = np.ones((cfg.d, cfg.d_ff), dtype=R)
    (a @ b)
    t1 = time.perf_counter()
    (a @ b)
    rate = 2.0 * 512 * cfg.d * cfg.d_ff / max(time.perf_counter() - t1, 1e-6)
    m = 3.0 if cfg.ffn == "swiglu" else 2.0
    per_row = 6.0 * m * cfg.d * cfg.d_ff                     # fwd + bwd FLOPs of one row of a routed expert
    per_row_sh = 6.0 * m * cfg.d * cfg.d_ff_shared
    active = [int(e) for e in np.argsort(counts, kind="stable") if counts[e] > 0]
    picks = [(active[0], None), (active[len(active) // 2], None)]
    room = budget_s * rate - sum(counts[e] for e, _ in picks) * per_row
    # the first shared expert and the largest routed expert get half of the budget each if they do not
    # fit whole; what is left goes to further whole experts, largest first
    n_sh = 0
    if cfg.n_shared:
        n_sh = int(min(cfg.T, max(64, 0.5 * room / per_row_sh)))
        room -= n_sh * per_row_sh
    for e in reversed(active[len(active) // 2 + 1:]):
        if e == active[-1]:
            cap = int(min(counts[e], max(64, room / per_row)))
            picks.append((e, None if cap == counts[e] else cap))
            room -= cap * per_row
        elif counts[e] * per_row <= room:
            picks.append((e, None))
            room -= counts[e] * per_row

    X = inp["X"].double().numpy()
    dY = inp["dY"].double().numpy()
    wide = lambda t: None if t is None else t.double().cpu().numpy()
    work = []
    for e, cap in picks:
        lo, hi = int(offsets[e]), int(offsets[e + 1])
        if cap is not None:
            hi = lo + cap
        a_ids = src_of[lo:hi]
        tok = a_ids // cfg.k
        work.append((X[tok], dY[tok] * w.reshape(-1)[a_ids][:, None], wide(weights["Wg"][e]),
                     wide(weights["Wu"][e]) if "Wu" in weights else None, wide(weights["Wd"][e]), per_row))
    if n_sh:
        work.append((X[:n_sh], dY[:n_sh], wide(weights["Wsg"][0]), wide(weights["Wsu"][0]) if "Wsu" in weights else None,
                     wide(weights["Wsd"][0]), per_row_sh))
    flops = 0.0
    t2 = time.perf_counter()
    for x, dy, Wg, Wu, Wd, pr in work:
        g, u, _, _ = orc.ffn(x, Wg, Wu, Wd)
        orc.ffn_bwd(x, Wg, Wu, Wd, g, u, dy)
        flops += x.shape[0] * pr
    dt = time.perf_counter() - t2
    total = cfg.flops()["total"]
    full_s = dt_plan + dt * total / flops
    rows = ", ".join(f"expert {e}: {counts[e] if cap is None else cap} of {counts[e]} rows" for e, cap in picks[:6])
    if len(picks) > 6:
        rows += f", and {len(picks) - 6} more whole experts of {sum(int(counts[e]) for e, _ in picks[6:])} rows"
    if n_sh:
        rows += f", shared expert 0: {n_sh} of {cfg.T} rows"
    return {"value": cfg.T / full_s, "unit": "tokens/s", "cores": blas_threads(), "kind": "oracle",
            "gflops": round(flops / dt / 1e9, 1), "sample_flops": flops, "sample_seconds": round(dt, 2),
            "host_cpus": os.cpu_count(),
            "sample": f"fp64 numpy oracle, fwd+bwd: route and dispatch plan of all {cfg.T} tokens ({dt_plan:.1f} s) plus the "
                      f"expert FFNs of whole experts ({rows}), {flops / 1e9:.0f} GFLOP in {dt:.1f} s, operands widened "
                      f"to fp64 beforehand; value = T / (plan time + sample time x total FLOPs / sample FLOPs)"}


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




def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", default="dsv3", choices=list(wl.CONFIGS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-overlap-shared", action="store_true",
                    help="keep the shared experts on the main stream in the timed region too (default: second stream)")
    ap.add_argument("--no-graph", action="store_true",
                    help="launch every kernel of the timed steps from the host (default: one captured HIP graph per step)")
    ap.add_argument("--gather", action="store_true",
                    help="routed experts read X and dY in place through src_of (moe_expert_*_gather)")
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
    hp = moe.MoEHotPath(shape, cfg.n_shared, cfg.d_ff_shared, dev, overlap_shared=not args.no_overlap_shared,
                        aux_alpha=cfg.aux_alpha, gather=args.gather)
    sh = [weights.get("Wsg"), weights.get("Wsu"), weights.get("Wsd")]

    def step():
        hp.forward(g["logits"], g["X"], weights["Wg"], weights.get("Wu"), weights["Wd"], *sh)
        hp.backward(g["dY"], g["X"], weights["Wg"], weights.get("Wu"), weights["Wd"], *sh)

    for _ in range(max(1, args.warmup)):
        step()
    torch.cuda.synchronize()
    sampled_err = verify(cfg, inp, weights, hp)
    # ---- the timed region: exactly `steps` bare steps (no per-kernel events), wall clock around all of
    # them, and one pair of HIP events per step on the launch stream for the median.  A step is the
    # same ~40 launches every time, so it is captured once into a HIP graph and replayed (the small
    # workloads are otherwise bound by the host's launch rate); the shared experts run on a second stream.
    run = step
    if not args.no_graph:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        run = graph.replay
        run()
        torch.cuda.synchronize()
        sampled_err = max(sampled_err, verify(cfg, inp, weights, hp))   # the replayed step, checked as well
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for a, b in ev:
        a.record()
        run()
        b.record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    step_ms = sorted(a.elapsed_time(b) for a, b in ev)
    median_ms = step_ms[len(step_ms) // 2] if len(step_ms) % 2 else 0.5 * (step_ms[len(step_ms) // 2 - 1] + step_ms[len(step_ms) // 2])

    # ---- a second, profiled pass of the same steps: the library brackets every launch with HIP events on
    # the launch stream (this costs a little time per launch, which is why it is not the headline)
    hp.overlap = False   # serial launches: the per-kernel durations then do not overlap
    moe.moe_profile_enable(True)
    t0p = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt_prof = time.perf_counter() - t0p

    # measured ceilings of this machine (outside the timed region).  One copy of known size: a profiler's HBM
    # counters are scaled by it.  One register-resident matrix loop: what the matrix pipe sustains.
    probe = torch.empty(2, PROBE_BYTES, dtype=torch.uint8, device=dev)
    probe.fill_(1)   # touches both halves, so that the copy is not timed on fresh pages
    for _ in range(PROBE_LAUNCHES):
        moe.moe_copy_probe(probe[0], probe[1])
    sink = torch.zeros(MFMA_PROBE_BLOCKS * 256, dtype=torch.float32, device=dev)
    mfma_flops = 0.0
    for _ in range(PROBE_LAUNCHES):
        mfma_flops = moe.moe_mfma_probe(MFMA_PROBE_BLOCKS, MFMA_PROBE_ITERS, sink)
    torch.cuda.synchronize()
    prof = moe.moe_profile_report()
    moe.moe_profile_enable(False)
    # cold-cache variant (outside the timed region, reported beside `value`): L2 and the infinity cache are
    # overwritten before every step by filling the 2 GiB probe buffer, and each step is timed on its own
    hp.overlap = bool(cfg.n_shared) and not args.no_overlap_shared
    cold = []
    for _ in range(COLD_STEPS):
        probe.fill_(2)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        run()
        torch.cuda.synchronize()
        cold.append(time.perf_counter() - t1)
    del probe
    probe_ms = prof.pop("copy_probe_kernel")[1] / PROBE_LAUNCHES
    # (mean of the launches: each lasts a few milliseconds, long enough for the clock to settle under the load)
    mfma_ms = prof.pop("mfma_probe_kernel")[1] / PROBE_LAUNCHES
    sustained_tf = mfma_flops / (mfma_ms * 1e-3) / 1e12

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
    # route, dispatch and combine kernels together: their algorithmic bytes over their summed time
    stream_ms = sum(kernels[l]["ms_per_step"] for l in kernels if l in byts or l.startswith("dispatch_"))
    stream_gbs = sum(byts.values()) / (stream_ms * 1e-3) / 1e9 if stream_ms > 0 else 0.0
    dom = max((l for l in GEMM_LABELS if l in kernels), key=lambda l: kernels[l]["ms_per_step"])
    dom_n, dom_ms = prof[dom]
    peak = MFMA_BF16_PEAK_TF if cfg.dtype == "bf16" else FP32_VEC_PEAK_TF
    achieved = flops[dom] * args.steps / (dom_ms * 1e-3) / 1e12
    dma_path = cfg.dtype == "bf16" and cfg.d % 64 == 0 and cfg.d_ff % 64 == 0   # SYMBOL names that path's kernels
    traffic, traffic_src = measured_traffic(cfg.name, SYMBOL[dom]) if dma_path else (None, None)
    roofline = {"bound": "mfma" if cfg.dtype == "bf16" else "alu", "kernel": dom, "symbol": SYMBOL[dom] if dma_path else None,
                "achieved": round(achieved, 2), "peak": peak, "unit": "TFLOP/s", "frac": round(achieved / peak, 4),
                "avg_launch_ms": round(dom_ms / dom_n, 4), "launches": dom_n,
                "flop_per_launch_avg": flops[dom] * args.steps / dom_n,
                "timing": "HIP events around every launch, on the launch stream, in a profiled pass of the same steps "
                          "right after the timed region",
                "traffic": traffic, "traffic_source": traffic_src}
    if cfg.dtype == "bf16":
        roofline["sustained_peak"] = round(sustained_tf, 1)   # register-resident matrix loop on this machine, same run
        roofline["frac_of_sustained"] = round(achieved / sustained_tf, 4)

    out = {
        "metric": "moe_layer_fwd_bwd_tokens_per_s", "value": round(cfg.T / (ms_per_step * 1e-3), 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "median_step_ms": round(median_ms, 4), "profiled_pass_ms_per_step": round(dt_prof / args.steps * 1e3, 4),
        "launch": {"hip_graph": not args.no_graph, "shared_experts_on_second_stream": bool(cfg.n_shared) and not args.no_overlap_shared,
                   "profiled_pass": "host launches, one stream, HIP events around every kernel"},
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: T={cfg.T} d={cfg.d} E={cfg.E} top-{cfg.k} {cfg.gate} d_ff={cfg.d_ff} "
                               f"shared={cfg.n_shared}x{cfg.d_ff_shared} routing={cfg.routing}(s={cfg.zipf_s}) seed={cfg.seed}",
                   "active_experts": int((counts > 0).sum()), "max_rows": int(counts.max()),
                   "load_share_std": round(float((counts.double() / counts.sum()).std(unbiased=False)), 5)},
        "grouped_gemm_tflops": round(gemm_tflops, 2), "grouped_gemm_frac_mfma_peak": round(gemm_tflops / peak, 4),
        "grouped_gemm_frac_of_sustained": round(gemm_tflops / sustained_tf, 4) if cfg.dtype == "bf16" else None,
        "streaming_gbs": round(stream_gbs, 1), "streaming_frac_hbm_peak": round(stream_gbs / HBM_PEAK_GBS, 4),
        "streaming_frac_of_copy_probe": round(stream_gbs / (2 * PROBE_BYTES / (probe_ms * 1e-3) / 1e9), 4),
        "total_tflops": round(cfg.flops()["total"] / (ms_per_step * 1e-3) / 1e12, 2),
        "cold_cache_ms_per_step": round(sum(cold) / len(cold) * 1e3, 4),
        "roofline": roofline, "kernels": kernels,
        "copy_probe": {"bytes_each_way": PROBE_BYTES, "ms": round(probe_ms, 4),
                       "gbs": round(2 * PROBE_BYTES / (probe_ms * 1e-3) / 1e9, 1)},
        "mfma_probe": {"flops_per_launch": mfma_flops, "ms": round(mfma_ms, 4), "tflops": round(sustained_tf, 1),
                       "frac_mfma_peak": round(sustained_tf / MFMA_BF16_PEAK_TF, 4)}, "sampled_error_vs_oracle": float(f"{sampled_err:.3e}"),
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, inp, weights)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
