"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element.

Integer outputs (top-k indices, counts, offsets, permutations, active ids) must be bit-exact.
Floating-point outputs must satisfy  max|gpu - ref| / max|ref| <= 1e-4 (fp32 path) or 2e-2 (bf16
path) per tensor, the tolerances BASELINE's north star states.
"""
import dataclasses

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import moe_oracle as orc

from .helpers import np64, oracle_inputs, problem, scale_rel_err, small_cfg

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}
INT_KEYS = ("topk_idx", "counts", "offsets", "row_of", "src_of")


def hot_path(cfg, gather=False):
    import paper_2502_02581_amd as moe

    shape = moe.MoEShape(cfg.T, cfg.d, cfg.E, cfg.k, cfg.d_ff, cfg.dtype, cfg.gate, cfg.renorm)
    return moe.MoEHotPath(shape, cfg.n_shared, cfg.d_ff_shared, aux_alpha=cfg.aux_alpha, gather=gather)


def run_gpu(cfg, p, gather=False):
    """One forward+backward on the GPU; returns the named buffers as CPU tensors."""
    hp = hot_path(cfg, gather)
    dev = hp.device
    g = {k: v.to(dev) for k, v in p.items()}
    shared = [g.get("Wsg"), g.get("Wsu"), g.get("Wsd")]
    hp.forward(g["logits"], g["X"], g["Wg"], g.get("Wu"), g["Wd"], *shared)
    hp.backward(g["dY"], g["X"], g["Wg"], g.get("Wu"), g["Wd"], *shared)
    torch.cuda.synchronize()
    return {k: v.cpu() for k, v in hp.b.items()}


def run_oracle(cfg, p):
    o = oracle_inputs(p)
    return orc.layer_fwd_bwd(o["logits"], o["X"], o["dY"], o["Wg"], o.get("Wu"), o["Wd"], cfg.k, cfg.gate, cfg.renorm,
                             o.get("Wsg"), o.get("Wsu"), o.get("Wsd"), want_dlogits=True, aux_alpha=cfg.aux_alpha)


def compare_layer(cfg, got, ref):
    tol = TOL[cfg.dtype]
    for key in INT_KEYS:
        assert np.array_equal(got[key].numpy().reshape(-1), np.asarray(ref[key]).reshape(-1)), key
    n_act = int(ref["n_active"])
    assert int(got["n_active"][0]) == n_act
    assert np.array_equal(got["active_ids"].numpy(), ref["active_ids"])
    errs = {}
    errs["topk_w"] = scale_rel_err(got["topk_w"], ref["topk_w"])
    assert errs["topk_w"] <= 1e-5
    gated = cfg.ffn == "swiglu"   # the two-matrix expert has no U, Wu, dWu
    fp = ["Xp", "G", "H", "Yp", "Y", "dYp", "dw", "dXp", "dX", "dlogits"] + (["U"] if gated else [])
    if cfg.n_shared:
        fp += ["Ysh", "dXsh", "dWsg", "dWsd"] + (["dWsu"] if gated else [])
    for key in fp:
        errs[key] = scale_rel_err(got[key], ref[key])
    if cfg.aux_alpha > 0:
        errs["aux_P"] = scale_rel_err(got["aux_P"], ref["aux_P"])
        assert abs(float(got["aux_loss"][0]) - ref["aux_loss"]) <= 1e-4 * abs(ref["aux_loss"])
    if cfg.n_shared:
        errs["Gs"] = scale_rel_err(got["Gs"], ref["Gs"])
        if gated:
            errs["Us"] = scale_rel_err(got["Us"], ref["Us"])
    ids = ref["active_ids"][:n_act]
    # per activated expert, each against the size of its own gradient: a light expert's gradient is
    # small beside the hottest one's and must not hide behind it
    for key in ("dWg", "dWu", "dWd") if gated else ("dWg", "dWd"):
        errs[key] = max((scale_rel_err(got[key + "_c"][i], ref[key][int(ids[i])]) for i in range(n_act)), default=0.0)
    bad = {k: v for k, v in errs.items() if not v <= tol}
    assert not bad, f"{cfg.name}: over tolerance {tol}: {bad}\nall: {errs}"
    # the dispatched rows are copies: exact
    assert errs["Xp"] == 0.0
    return errs


LAYER_CASES = [
    # fp32 path: several 64-row tiles per expert, ragged tails, K not a multiple of the K tile
    (small_cfg("f32-a", T=300, d=72, E=6, k=2, d_ff=104, dtype="f32", zipf_s=1.0), True),
    (small_cfg("f32-sig", T=130, d=40, E=9, k=3, d_ff=56, dtype="f32", gate="sigmoid", zipf_s=1.5, n_shared=2,
               d_ff_shared=24), True),
    (small_cfg("f32-norenorm", T=64, d=32, E=5, k=2, d_ff=48, dtype="f32", renorm=False), True),
    # auxiliary loss with a weight large enough for its share of dlogits to show at the tolerance
    (small_cfg("f32-aux", T=300, d=72, E=6, k=2, d_ff=104, dtype="f32", zipf_s=1.0, aux_alpha=3000.0), True),
    (small_cfg("bf16-aux-sig", T=400, d=192, E=20, k=4, d_ff=72, dtype="bf16", gate="sigmoid", zipf_s=1.5,
               n_shared=1, d_ff_shared=136, aux_alpha=3000.0), True),
    # two-matrix GELU experts (Eq. 1 as printed): fp32 path, general bf16 path, LDS-DMA path with tall
    # tiles and ragged remainders, with shared experts, and the top-k sweep of the paper (2..5)
    (small_cfg("f32-gelu", T=300, d=72, E=6, k=2, d_ff=104, dtype="f32", zipf_s=1.0, ffn="gelu"), True),
    (small_cfg("bf16-gelu", T=700, d=136, E=6, k=2, d_ff=200, dtype="bf16", zipf_s=1.0, ffn="gelu"), True),
    (small_cfg("bf16-gelu-dma", T=1500, d=512, E=3, k=2, d_ff=384, dtype="bf16", zipf_s=0.5, ffn="gelu"), True),
    (small_cfg("bf16-gelu-shared", T=620, d=128, E=12, k=3, d_ff=192, dtype="bf16", zipf_s=1.3, ffn="gelu",
               n_shared=1, d_ff_shared=128), True),
    (small_cfg("bf16-gelu-k4", T=512, d=192, E=16, k=4, d_ff=256, dtype="bf16", zipf_s=1.0, ffn="gelu"), False),
    (small_cfg("bf16-gelu-k5", T=512, d=192, E=16, k=5, d_ff=256, dtype="bf16", zipf_s=1.0, ffn="gelu"), True),
    # bf16 MFMA path: 128-row tiles with ragged tails in M, N and K
    (small_cfg("bf16-a", T=700, d=136, E=6, k=2, d_ff=200, dtype="bf16", zipf_s=1.0), True),
    (small_cfg("bf16-paper-scale", T=700, d=136, E=6, k=2, d_ff=200, dtype="bf16", zipf_s=1.0), False),
    (small_cfg("bf16-sig-shared", T=400, d=192, E=20, k=4, d_ff=72, dtype="bf16", gate="sigmoid", zipf_s=1.5,
               n_shared=2, d_ff_shared=136), True),
    (small_cfg("bf16-many-empty", T=40, d=64, E=64, k=2, d_ff=64, dtype="bf16", zipf_s=2.5), True),
    (small_cfg("bf16-E1", T=200, d=64, E=1, k=1, d_ff=128, dtype="bf16"), True),
    (small_cfg("bf16-kE", T=96, d=64, E=4, k=4, d_ff=64, dtype="bf16"), True),
    # full 256-row tiles with several K iterations, ragged remainders of every tile height
    (small_cfg("bf16-big-tiles", T=1500, d=512, E=3, k=2, d_ff=384, dtype="bf16", zipf_s=0.5), True),
    (small_cfg("bf16-big-shared", T=700, d=256, E=2, k=1, d_ff=256, dtype="bf16", zipf_s=0.3, n_shared=1,
               d_ff_shared=320), True),
    (small_cfg("bf16-heights", T=620, d=128, E=12, k=3, d_ff=192, dtype="bf16", zipf_s=1.3, gate="sigmoid"), False),
    (small_cfg("bf16-stress", T=512, d=128, E=24, k=4, d_ff=96, dtype="bf16", routing="stress", zipf_s=1.5,
               ), True),
]


# odd multiples of 64 in d and d_ff (ragged last column tile and K counts that are not a multiple of the
# pipeline depth), a single token, fewer tokens than experts, shared experts of another width
SWEEP = [
    small_cfg("sw-1tok", T=1, d=64, E=4, k=2, d_ff=192, dtype="bf16"),
    small_cfg("sw-77", T=77, d=192, E=7, k=3, d_ff=64, dtype="bf16", zipf_s=1.0, gate="sigmoid"),
    small_cfg("sw-513", T=513, d=320, E=5, k=2, d_ff=448, dtype="bf16", zipf_s=0.7, n_shared=1, d_ff_shared=192),
    small_cfg("sw-wide", T=300, d=448, E=3, k=1, d_ff=320, dtype="bf16", zipf_s=2.0),
    small_cfg("sw-k1tail", T=260, d=576, E=2, k=2, d_ff=128, dtype="bf16", renorm=False),
    small_cfg("sw-fewtok", T=5, d=128, E=16, k=4, d_ff=128, dtype="bf16", n_shared=2, d_ff_shared=64),
]


@pytest.mark.parametrize("cfg", SWEEP, ids=lambda c: c.name)
def test_dma_path_shape_sweep(cfg):
    p = problem(cfg, unit_scale=True)
    errs = compare_layer(cfg, run_gpu(cfg, p), run_oracle(cfg, p))
    print(cfg.name, {k: f"{v:.2e}" for k, v in errs.items()})


@pytest.mark.parametrize("cfg,unit", LAYER_CASES, ids=lambda v: v.name if hasattr(v, "name") else str(v))
def test_layer_parity_small(cfg, unit):
    if cfg.routing == "stress":
        cfg = dataclasses.replace(cfg, n_zero=5)
    p = problem(cfg, unit_scale=unit)
    got = run_gpu(cfg, p)
    ref = run_oracle(cfg, p)
    errs = compare_layer(cfg, got, ref)
    print(cfg.name, {k: f"{v:.2e}" for k, v in errs.items()})


def test_config_tiny_full():
    """BASELINE config 1 in full: T=256, d=128, E=8, top-2, d_ff=256, fp32, seed 0."""
    cfg = wl.CONFIGS["tiny"]
    p = problem(cfg, unit_scale=False)
    errs = compare_layer(cfg, run_gpu(cfg, p), run_oracle(cfg, p))
    print({k: f"{v:.2e}" for k, v in errs.items()})


REDUCED = {
    # the four bf16 workloads with T and the widths cut so that the oracle finishes in seconds;
    # routing recipe, E, k, gate and shared experts as in the full configs
    "qwen": dict(T=1024, d=256, d_ff=192, d_ff_shared=192),
    "phi": dict(T=1536, d=256, d_ff=320),
    "dsv3": dict(T=768, d=256, d_ff=128, d_ff_shared=128),
    "stress": dict(T=2048, d=128, d_ff=96),
}


@pytest.mark.parametrize("name", list(REDUCED))
def test_configs_reduced(name):
    cfg = wl.scaled(wl.CONFIGS[name], **REDUCED[name])
    for unit in (False, True):
        p = problem(cfg, unit_scale=unit)
        errs = compare_layer(cfg, run_gpu(cfg, p), run_oracle(cfg, p))
        print(name, unit, {k: f"{v:.2e}" for k, v in errs.items()})


GATHER_CASES = ["f32-sig", "f32-gelu", "bf16-a", "bf16-gelu", "bf16-sig-shared", "bf16-many-empty", "bf16-big-tiles",
                "bf16-heights", "bf16-stress", "bf16-gelu-dma", "bf16-kE"]


@pytest.mark.parametrize("name", GATHER_CASES)
def test_gathered_expert_calls(name):
    """moe_expert_fwd_gather / moe_expert_bwd_gather (token rows read in place through src_of) against the
    oracle, on all three GEMM paths; the forward products read the same values in the same order as the
    calls on permuted copies, so G, U, H and Yp must come out with identical bits."""
    cfg, unit = next((c, u) for c, u in LAYER_CASES if c.name == name)
    if cfg.routing == "stress":
        cfg = dataclasses.replace(cfg, n_zero=5)
    p = problem(cfg, unit_scale=unit)
    got = run_gpu(cfg, p, gather=True)
    plain = run_gpu(cfg, p, gather=False)
    for key in ("G", "H", "Yp", "Y") + (("U",) if cfg.ffn == "swiglu" else ()):
        assert torch.equal(got[key].view(torch.uint8), plain[key].view(torch.uint8)), key
    errs = compare_layer(cfg, got, run_oracle(cfg, p))
    print(cfg.name, {k: f"{v:.2e}" for k, v in errs.items()})


def test_gathered_reduced_dsv3():
    cfg = wl.scaled(wl.CONFIGS["dsv3"], **REDUCED["dsv3"])
    for unit in (False, True):
        p = problem(cfg, unit_scale=unit)
        compare_layer(cfg, run_gpu(cfg, p, gather=True), run_oracle(cfg, p))


# ------------------------------------------------------------------- single entry points
def test_route_ties_and_masks():
    import paper_2502_02581_amd as moe

    E, k = 70, 5
    lg = torch.zeros(6, E)
    lg[1, 10:20] = 1.0          # ten-way tie at the top
    lg[2] = -1.0e4
    lg[2, 65] = 3.0
    lg[3] = torch.arange(E, dtype=torch.float32)
    lg[4] = -torch.arange(E, dtype=torch.float32)
    lg[5, ::7] = 2.5
    for gate in ("softmax", "sigmoid"):
        for renorm in (True, False):
            shape = moe.MoEShape(6, 8, E, k, 8, "f32", gate, renorm)
            idx = torch.empty(6, k, dtype=torch.int32, device="cuda")
            w = torch.empty(6, k, dtype=torch.float32, device="cuda")
            moe.moe_route(shape, lg.cuda(), idx, w)
            ridx, rw = orc.route(lg.numpy(), k, gate, renorm)
            assert np.array_equal(idx.cpu().numpy(), ridx)
            np.testing.assert_allclose(w.cpu().numpy(), rw, rtol=1e-5, atol=1e-30)


def _bf16_nearest_even(x32: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns of fp32 values, from the definition: the nearer of the two neighbouring
    bfloat16 values (exact comparison in fp64), the one with an even last bit on a tie."""
    u = x32.view(np.uint32).astype(np.uint64)
    lo = u & 0xFFFF0000                       # towards zero
    hi = lo + 0x10000                         # away from zero (may carry into the exponent: that is the next value)
    f = lambda b: b.astype(np.uint32).view(np.float32).astype(np.float64)
    x = x32.astype(np.float64)
    with np.errstate(invalid="ignore", over="ignore"):
        d_lo, d_hi = np.abs(x - f(lo)), np.abs(f(hi) - x)
        # past the largest finite bfloat16 the upper neighbour is infinity, whose distance is measured
        # to the value the format would have there (2^128)
        top = (lo & 0x7FFF0000) == 0x7F7F0000
        d_hi = np.where(top, np.abs(np.ldexp(1.0, 128) - np.abs(x)), d_hi)
    take_hi = (d_hi < d_lo) | ((d_hi == d_lo) & ((lo >> 16) & 1 == 1))
    out = np.where(take_hi, hi, lo) >> 16
    return out.astype(np.uint16)


def test_bf16_rounding_is_nearest_even():
    """The bf16 outputs are rounded by the conversion instruction of the chip; pin its rounding, bit for
    bit, through the combine kernel: one token per value, top-1, a row of ones, weight = the value."""
    import paper_2502_02581_amd as moe

    rng = np.random.default_rng(11)
    # (no -0.0: the kernel adds the product to a sum that starts at +0)
    special = np.array([0.0, 1.0, -1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20,
                        1.0 + 2.0 ** -7, 1.0 - 2.0 ** -9, 3.3895314e38, 3.3961775e38, 3.4e38, -3.4e38, np.inf, -np.inf,
                        1e-38, 1.1754944e-38, 5.877e-39, 1e-40, 9.18e-41, 4.6e-41, 1e-45, 65504.0, 0.1, -0.3, 1 / 3],
                       dtype=np.float32)
    bits = rng.integers(0, 2 ** 32, size=4096 - len(special), dtype=np.uint64).astype(np.uint32)
    vals = np.concatenate([special, bits.view(np.float32)])
    vals = vals[~np.isnan(vals)]
    T = len(vals)
    shape = moe.MoEShape(T, 8, 4, 1, 8, "bf16")
    Yp = torch.ones(T, 8, dtype=torch.bfloat16, device="cuda")
    row_of = torch.arange(T, dtype=torch.int32, device="cuda").reshape(T, 1)
    w = torch.from_numpy(vals.copy()).reshape(T, 1).cuda()
    Y = torch.zeros(T, 8, dtype=torch.bfloat16, device="cuda")
    moe.moe_combine(shape, Yp, row_of, w, None, Y)
    got = Y.cpu().view(torch.int16).numpy().view(np.uint16)
    want = _bf16_nearest_even(vals)
    assert np.array_equal(got, np.repeat(want[:, None], 8, axis=1)), \
        [(float(v), hex(int(g)), hex(int(e))) for v, g, e in zip(vals, got[:, 0], want) if g != e][:8]
    # NaN stays NaN
    wn = torch.full((T, 1), float("nan"), device="cuda")
    moe.moe_combine(shape, Yp, row_of, wn, None, Y)
    assert bool(torch.isnan(Y.float()).all())


@pytest.mark.parametrize("E,k", [(1, 1), (8, 8), (64, 3), (65, 2), (256, 8), (300, 6), (1024, 64)])
def test_route_dispatch_shapes(E, k):
    import paper_2502_02581_amd as moe

    T = 517
    cfg = small_cfg(T=T, d=8, E=E, k=k, d_ff=8, zipf_s=1.2, seed=3)
    lg = wl.make_logits(cfg)
    shape = moe.MoEShape(T, 8, E, k, 8, "f32")
    dev = "cuda"
    idx = torch.empty(T, k, dtype=torch.int32, device=dev)
    w = torch.empty(T, k, dtype=torch.float32, device=dev)
    moe.moe_route(shape, lg.to(dev), idx, w)
    ridx, rw = orc.route(lg.numpy(), k)
    assert np.array_equal(idx.cpu().numpy(), ridx)
    np.testing.assert_allclose(w.cpu().numpy(), rw, rtol=2e-5)
    X = wl.make_tokens(cfg).to(dev)
    out = {n: torch.empty(s, dtype=torch.int32, device=dev) for n, s in
           (("counts", E), ("offsets", E + 1), ("row_of", T * k), ("src_of", T * k))}
    Xp = torch.empty(T * k, 8, device=dev)
    ws = torch.empty(moe.moe_dispatch_workspace_bytes(shape), dtype=torch.uint8, device=dev)
    moe.moe_dispatch(shape, X, idx, out["counts"], out["offsets"], out["row_of"], out["src_of"], Xp, ws)
    ref = orc.dispatch_plan(ridx, E)
    for got, exp in zip(("counts", "offsets", "row_of", "src_of"), ref):
        assert np.array_equal(out[got].cpu().numpy(), exp), got
    assert torch.equal(Xp.cpu(), X.cpu()[torch.arange(T * k) // k][torch.from_numpy(ref[3]).long()])


@pytest.mark.parametrize("E,k", [(1, 1), (8, 8), (64, 3), (65, 2), (256, 8), (300, 6), (1024, 64)])
@pytest.mark.parametrize("gate", ["softmax", "sigmoid"])
@pytest.mark.parametrize("renorm", [True, False])
def test_route_bwd(E, k, gate, renorm):
    """Gradient of the router logits from given dw, against the oracle's route_bwd (fp32 arithmetic: 1e-4)."""
    import paper_2502_02581_amd as moe

    T = 203
    cfg = small_cfg(T=T, d=8, E=E, k=k, d_ff=8, zipf_s=1.2, seed=5)
    lg = wl.make_logits(cfg)
    dw = torch.randn(T, k, generator=torch.Generator().manual_seed(11))
    shape = moe.MoEShape(T, 8, E, k, 8, "f32", gate, renorm)
    ridx, _ = orc.route(lg.numpy(), k, gate, renorm)
    ref = orc.route_bwd(lg.numpy(), ridx, dw.numpy(), gate, renorm)
    out = torch.full((T, E), float("nan"), device="cuda")
    moe.moe_route_bwd(shape, lg.cuda(), torch.from_numpy(ridx).cuda(), dw.cuda(), out)
    assert scale_rel_err(out.cpu(), ref) <= 1e-4


@pytest.mark.parametrize("T,E,k", [(1, 1, 1), (5, 64, 1), (203, 40, 3), (300, 65, 2), (1500, 256, 8), (2100, 300, 6),
                                   (8192, 256, 8), (77, 1024, 64)])
@pytest.mark.parametrize("gate", ["softmax", "sigmoid"])
def test_aux_loss(T, E, k, gate):
    """Auxiliary load-balancing loss, its per-expert mean shares and its gradient (written and accumulated)
    against the oracle (fp32 arithmetic: 1e-4), with counts taken from the oracle's dispatch plan; the
    partial sums are reduced in a fixed order, so a second run gives identical bits."""
    import paper_2502_02581_amd as moe

    cfg = small_cfg(T=T, d=8, E=E, k=k, d_ff=8, zipf_s=1.2, seed=9)
    lg = wl.make_logits(cfg)
    shape = moe.MoEShape(T, 8, E, k, 8, "f32", gate, True)
    ridx, _ = orc.route(lg.numpy(), k, gate, True)
    counts = orc.dispatch_plan(ridx, E)[0]
    alpha, dloss = 0.01, 1.7
    L_ref, P_ref = orc.aux_loss(lg.numpy(), counts, k, alpha, gate)
    g_ref = orc.aux_loss_bwd(lg.numpy(), counts, k, alpha, gate, dloss)
    dev = "cuda"
    ws = torch.empty(moe.moe_aux_loss_workspace_bytes(shape), dtype=torch.uint8, device=dev)
    c_dev = torch.from_numpy(counts).to(dev)
    runs = []
    for _ in range(2):
        P = torch.full((E,), float("nan"), device=dev)
        L = torch.full((1,), float("nan"), device=dev)
        ws.fill_(255)
        moe.moe_aux_loss(shape, lg.to(dev), c_dev, alpha, P, L, ws)
        runs.append((P.cpu(), L.cpu()))
    assert torch.equal(runs[0][0], runs[1][0]) and torch.equal(runs[0][1], runs[1][1])
    assert scale_rel_err(runs[0][0], P_ref) <= 1e-4
    assert abs(float(runs[0][1]) - L_ref) <= 1e-4 * abs(L_ref)
    out = torch.full((T, E), float("nan"), device=dev)
    moe.moe_aux_loss_bwd(shape, lg.to(dev), c_dev, alpha, dloss, False, out)
    assert scale_rel_err(out.cpu(), g_ref) <= 1e-4
    base = torch.randn(T, E, generator=torch.Generator().manual_seed(2)) * float(np.abs(g_ref).max())
    acc = base.to(dev)
    moe.moe_aux_loss_bwd(shape, lg.to(dev), c_dev, alpha, dloss, True, acc)
    assert scale_rel_err(acc.cpu(), base.double().numpy() + g_ref) <= 1e-4


def test_aux_loss_empty_batch():
    import paper_2502_02581_amd as moe

    shape = moe.MoEShape(0, 8, 6, 2, 8, "f32")
    P = torch.full((6,), 5.0, device="cuda")
    L = torch.full((1,), 5.0, device="cuda")
    ws = torch.empty(max(1, moe.moe_aux_loss_workspace_bytes(shape)), dtype=torch.uint8, device="cuda")
    moe.moe_aux_loss(shape, None, None, 0.01, P, L, ws)
    moe.moe_aux_loss_bwd(shape, None, None, 0.01, 1.0, False, None)
    assert not P.cpu().any() and float(L) == 0.0


ROUTER_CASES = [
    # (T, d, E, dtype): fp32 path; general bf16 path (d not a multiple of 64); LDS-DMA path with E
    # not a multiple of 8, E a multiple of 64, E above one column tile
    (70, 40, 6, "f32"), (300, 72, 60, "f32"), (130, 136, 12, "bf16"), (513, 192, 60, "bf16"),
    (700, 256, 64, "bf16"), (1100, 448, 320, "bf16"), (1, 64, 1, "bf16"),
]


@pytest.mark.parametrize("T,d,E,dtype", ROUTER_CASES)
def test_router_linear_map(T, d, E, dtype):
    """logits = X Wr, dWr = X^T dlogits, dX (+)= dlogits Wr^T against the oracle."""
    import paper_2502_02581_amd as moe

    g = torch.Generator().manual_seed(17)
    td = torch.float32 if dtype == "f32" else torch.bfloat16
    X = torch.randn(T, d, generator=g).to(td)
    Wr = (torch.randn(d, E, generator=g) / d ** 0.5).to(td)
    dl = torch.randn(T, E, generator=g)
    dX0 = torch.randn(T, d, generator=g).to(td)
    shape = moe.MoEShape(T, d, E, 1, 64, dtype)
    dev = "cuda"
    ws = torch.empty(max(moe.moe_router_fwd_workspace_bytes(shape), moe.moe_router_bwd_workspace_bytes(shape)),
                     dtype=torch.uint8, device=dev)
    logits = torch.full((T, E), float("nan"), device=dev)
    moe.moe_router_fwd(shape, X.to(dev), Wr.to(dev), logits, ws)
    ref = orc.router_fwd(np64(X), np64(Wr))
    assert scale_rel_err(logits.cpu(), ref) <= 1e-4  # fp32 output of exactly representable operands
    tol = TOL[dtype]
    ref_dX, ref_dWr = orc.router_bwd(np64(X), np64(Wr), dl.numpy())
    for accumulate in (False, True):
        dWr = torch.full((d, E), float("nan"), dtype=td, device=dev)
        dX = dX0.to(dev).clone()
        moe.moe_router_bwd(shape, X.to(dev), Wr.to(dev), dl.to(dev), dWr, dX, accumulate, ws)
        assert scale_rel_err(dWr.cpu(), ref_dWr) <= tol
        assert scale_rel_err(dX.cpu(), ref_dX + (np64(dX0) if accumulate else 0.0)) <= tol


def test_overlap_shared_is_identical():
    """Shared experts on a second stream: bit-identical to the single-stream order."""
    import paper_2502_02581_amd as moe

    cfg = small_cfg("ovl", T=700, d=256, E=4, k=2, d_ff=256, dtype="bf16", zipf_s=0.8, n_shared=2, d_ff_shared=192)
    p = problem(cfg)
    g = {k: v.cuda() for k, v in p.items()}
    shape = moe.MoEShape(cfg.T, cfg.d, cfg.E, cfg.k, cfg.d_ff, cfg.dtype, cfg.gate, cfg.renorm)
    outs = []
    for overlap in (False, True):
        hp = moe.MoEHotPath(shape, cfg.n_shared, cfg.d_ff_shared, "cuda:0", overlap_shared=overlap, aux_alpha=cfg.aux_alpha)
        for _ in range(3):  # repeated steps reuse the buffers and the events
            hp.forward(g["logits"], g["X"], g["Wg"], g["Wu"], g["Wd"], g["Wsg"], g["Wsu"], g["Wsd"])
            hp.backward(g["dY"], g["X"], g["Wg"], g["Wu"], g["Wd"], g["Wsg"], g["Wsu"], g["Wsd"])
        torch.cuda.synchronize()
        outs.append({k: hp.b[k].cpu() for k in ("Y", "dX", "dw", "dlogits", "dWsg", "dWsu", "dWsd", "Ysh", "dXsh")})
    for k in outs[0]:
        assert torch.equal(outs[0][k], outs[1][k]), k


def test_determinism():
    """Two runs give bit-identical outputs, floating point included (no atomics on fp data)."""
    cfg = wl.scaled(wl.CONFIGS["stress"], T=1024, d=128, d_ff=96)
    p = problem(cfg)
    a = run_gpu(cfg, p)
    b = run_gpu(cfg, p)
    n_act = int(a["n_active"][0])
    for k, v in a.items():
        if k in ("dWg_c", "dWu_c", "dWd_c"):
            assert torch.equal(v[:n_act], b[k][:n_act]), k
        else:
            assert torch.equal(v, b[k]), k


def test_empty_batch():
    """T = 0: every call succeeds, counts/offsets/n_active are written (zeros), nothing else is touched."""
    import paper_2502_02581_amd as moe

    for dtype in ("f32", "bf16"):
        cfg = small_cfg("empty", T=0, d=64, E=5, k=2, d_ff=64, dtype=dtype, n_shared=1, d_ff_shared=64)
        W = wl.make_weights(cfg, "cuda")
        shape = moe.MoEShape(0, cfg.d, cfg.E, cfg.k, cfg.d_ff, cfg.dtype, cfg.gate, cfg.renorm)
        hp = moe.MoEHotPath(shape, cfg.n_shared, cfg.d_ff_shared, "cuda:0")
        for key in ("counts", "offsets", "n_active", "active_ids"):
            hp.b[key].fill_(77)
        hp.b["dWg_c"].fill_(3.0)
        x = torch.empty(0, cfg.d, dtype=shape.torch_dtype, device="cuda")
        lg = torch.empty(0, cfg.E, device="cuda")
        y = hp.forward(lg, x, W["Wg"], W["Wu"], W["Wd"], W["Wsg"], W["Wsu"], W["Wsd"])
        dx = hp.backward(x, x, W["Wg"], W["Wu"], W["Wd"], W["Wsg"], W["Wsu"], W["Wsd"])
        torch.cuda.synchronize()
        assert y.shape == (0, cfg.d) and dx.shape == (0, cfg.d)
        assert not hp.b["counts"].any() and not hp.b["offsets"].any()
        assert int(hp.b["n_active"].item()) == 0 and bool((hp.b["active_ids"] == -1).all())
        assert bool((hp.b["dWg_c"] == 3.0).all())  # no expert is active: no gradient slot is written


def test_error_paths_launch_nothing():
    import paper_2502_02581_amd as moe

    shape = moe.MoEShape(4, 12, 4, 2, 8, "f32")  # d not a multiple of 8
    t = torch.zeros(64, device="cuda")
    i = torch.zeros(64, dtype=torch.int32, device="cuda")
    with pytest.raises(moe.MoEError, match="multiples of 8"):
        moe.moe_route(shape, t, i, t)
    shape = moe.MoEShape(4, 8, 4, 5, 8, "f32")  # k > E
    with pytest.raises(moe.MoEError, match="bad shape"):
        moe.moe_route(shape, t, i, t)
    shape = moe.MoEShape(4, 8, 4, 2, 8, "f32")
    ws = torch.zeros(8, dtype=torch.uint8, device="cuda")
    with pytest.raises(moe.MoEError, match="workspace"):
        moe.moe_dispatch(shape, t, i, i, i, i, i, t, ws)
    with pytest.raises(moe.MoEError, match="GPU"):
        moe.moe_route(shape, torch.zeros(16), i, t)


# ------------------------------------------------------------------- memory the path does not own
GUARD = 4096  # bytes on either side of every buffer
FILL = 0xA5


def _guarded(t: torch.Tensor):
    """A tensor of the same shape and dtype inside a larger byte buffer filled with FILL."""
    n = t.numel() * t.element_size()
    big = torch.full((n + 2 * GUARD,), FILL, dtype=torch.uint8, device=t.device)
    return big, big[GUARD:GUARD + n].view(t.dtype).view(t.shape)


@pytest.mark.parametrize("cfg", [
    small_cfg("guard-f32", T=130, d=40, E=9, k=3, d_ff=56, dtype="f32", gate="sigmoid", zipf_s=1.5, n_shared=2, d_ff_shared=24),
    small_cfg("guard-bf16", T=700, d=136, E=6, k=2, d_ff=200, dtype="bf16", zipf_s=1.0),
    small_cfg("guard-dma-empty", T=40, d=64, E=64, k=2, d_ff=64, dtype="bf16", zipf_s=2.5, aux_alpha=0.001),
    small_cfg("guard-dma-tiles", T=1500, d=512, E=5, k=2, d_ff=384, dtype="bf16", zipf_s=2.0, n_shared=1, d_ff_shared=192),
], ids=lambda c: c.name)
def test_nothing_outside_the_outputs_is_written(cfg):
    """Every buffer the path writes (outputs, saved activations, workspaces) sits between guard bands, and
    the compact weight-gradient buffers are pre-filled: after a normal forward+backward the bands and the
    slots at and beyond n_active still hold the fill pattern, byte for byte."""
    p = problem(cfg, unit_scale=True)
    hp = hot_path(cfg)
    keep = []
    for key in list(hp.b):
        big, view = _guarded(hp.b[key])
        keep.append((key, big))
        hp.b[key] = view
    big_ws, hp.ws = _guarded(hp.ws)
    hp.ws_shared = hp.ws
    keep.append(("ws", big_ws))
    g = {k: v.to(hp.device) for k, v in p.items()}
    shared = [g.get("Wsg"), g.get("Wsu"), g.get("Wsd")]
    hp.forward(g["logits"], g["X"], g["Wg"], g.get("Wu"), g["Wd"], *shared)
    hp.backward(g["dY"], g["X"], g["Wg"], g.get("Wu"), g["Wd"], *shared)
    torch.cuda.synchronize()
    for key, big in keep:
        assert bool((big[:GUARD] == FILL).all()) and bool((big[-GUARD:] == FILL).all()), f"guard band of {key} was written"
    n_act = int(hp.b["n_active"].item())
    assert 0 < n_act <= cfg.E
    for key in ("dWg_c", "dWu_c", "dWd_c"):
        tail = hp.b[key][n_act:].contiguous().view(torch.uint8)
        assert bool((tail == FILL).all()), f"{key}: a slot at or beyond n_active was written"
    # and the result is still the right one
    ref = run_oracle(cfg, p)
    compare_layer(cfg, {k: v.cpu() for k, v in hp.b.items()}, ref)


def test_step_replayed_from_a_hip_graph():
    """One forward+backward captured into a HIP graph (the shared experts on a second stream, as the
    benchmark launches it) and replayed several times, with eager steps on other inputs and
    synchronisations in between: every replay must reproduce the eager result bit for bit."""
    import paper_2502_02581_amd as moe

    cfg = small_cfg("graph", T=620, d=128, E=12, k=3, d_ff=192, dtype="bf16", zipf_s=1.3, gate="sigmoid", n_shared=1,
                    d_ff_shared=128, aux_alpha=0.001)
    p = problem(cfg, unit_scale=True)
    shape = moe.MoEShape(cfg.T, cfg.d, cfg.E, cfg.k, cfg.d_ff, cfg.dtype, cfg.gate, cfg.renorm)
    hp = moe.MoEHotPath(shape, cfg.n_shared, cfg.d_ff_shared, overlap_shared=True, aux_alpha=cfg.aux_alpha)
    g = {k: v.to(hp.device) for k, v in p.items()}
    other = {k: (v.clone().normal_() if v.is_floating_point() else v) for k, v in g.items()}
    sh = lambda q: [q.get("Wsg"), q.get("Wsu"), q.get("Wsd")]

    def step(q):
        hp.forward(q["logits"], q["X"], q["Wg"], q.get("Wu"), q["Wd"], *sh(q))
        hp.backward(q["dY"], q["X"], q["Wg"], q.get("Wu"), q["Wd"], *sh(q))

    keys = ("topk_idx", "row_of", "Y", "dX", "dw", "dlogits", "dWg_c", "dWd_c", "dWsg", "aux_loss")
    step(g)
    torch.cuda.synchronize()
    eager = {k: hp.b[k].clone() for k in keys}
    n_act = int(hp.b["n_active"].item())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step(g)
    for rep in range(4):
        step(other)                      # eager work of the program itself between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k in keys:
            a, b = hp.b[k], eager[k]
            if k in ("dWg_c", "dWd_c"):
                a, b = a[:n_act], b[:n_act]
            assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), (rep, k)


@pytest.mark.parametrize("T,E,k", [(1, 1, 1), (517, 8, 8), (517, 64, 3), (300, 65, 2), (1500, 256, 8), (2100, 300, 6),
                                   (8192, 256, 8), (77, 1024, 64), (1000, 60, 5)])
@pytest.mark.parametrize("gate", ["softmax", "sigmoid"])
def test_fused_prologue_matches_separate_calls(T, E, k, gate):
    """moe_route_dispatch against moe_route + moe_dispatch + moe_aux_loss, and moe_route_aux_bwd against
    moe_route_bwd + moe_aux_loss_bwd: integers, combine weights and copied rows bit for bit, the loss terms
    to fp32 summation order; everything against the oracle as well."""
    import paper_2502_02581_amd as moe

    cfg = small_cfg(T=T, d=16, E=E, k=k, d_ff=8, zipf_s=1.2, seed=13, dtype="bf16")
    lg = wl.make_logits(cfg)
    shape = moe.MoEShape(T, 16, E, k, 8, "bf16", gate, True)
    dev = "cuda"
    alpha = 0.01
    X = wl.make_tokens(cfg).to(dev)
    lgd = lg.to(dev)

    def bufs():
        i32 = dict(dtype=torch.int32, device=dev)
        return {"topk_idx": torch.full((T, k), -3, **i32), "topk_w": torch.full((T, k), float("nan"), device=dev),
                "counts": torch.full((E,), -3, **i32), "offsets": torch.full((E + 1,), -3, **i32),
                "row_of": torch.full((T * k,), -3, **i32), "src_of": torch.full((T * k,), -3, **i32),
                "Xp": torch.full((T * k, 16), float("nan"), dtype=torch.bfloat16, device=dev),
                "P": torch.full((E,), float("nan"), device=dev), "L": torch.full((1,), float("nan"), device=dev)}

    a, b = bufs(), bufs()
    ws = torch.empty(max(moe.moe_dispatch_workspace_bytes(shape), moe.moe_aux_loss_workspace_bytes(shape),
                         moe.moe_route_dispatch_workspace_bytes(shape)), dtype=torch.uint8, device=dev)
    moe.moe_route(shape, lgd, a["topk_idx"], a["topk_w"])
    moe.moe_dispatch(shape, X, a["topk_idx"], a["counts"], a["offsets"], a["row_of"], a["src_of"], a["Xp"], ws)
    moe.moe_aux_loss(shape, lgd, a["counts"], alpha, a["P"], a["L"], ws)
    ws.fill_(255)
    moe.moe_route_dispatch(shape, lgd, X, alpha, b["topk_idx"], b["topk_w"], b["counts"], b["offsets"], b["row_of"],
                           b["src_of"], b["Xp"], b["P"], b["L"], ws)
    torch.cuda.synchronize()
    for key in ("topk_idx", "topk_w", "counts", "offsets", "row_of", "src_of", "Xp"):
        assert torch.equal(a[key].view(torch.uint8), b[key].view(torch.uint8)), key
    ridx, rw = orc.route(lg.numpy(), k, gate, True)
    assert np.array_equal(b["topk_idx"].cpu().numpy(), ridx)
    rc = orc.dispatch_plan(ridx, E)
    assert np.array_equal(b["counts"].cpu().numpy(), rc[0]) and np.array_equal(b["row_of"].cpu().numpy(), rc[2])
    L_ref, P_ref = orc.aux_loss(lg.numpy(), rc[0], k, alpha, gate)
    assert scale_rel_err(b["P"].cpu(), P_ref) <= 1e-4 and scale_rel_err(a["P"].cpu(), P_ref) <= 1e-4
    assert abs(float(b["L"].item()) - L_ref) <= 1e-4 * abs(L_ref)
    # without the loss: P and L are not touched
    c = bufs()
    moe.moe_route_dispatch(shape, lgd, X, 0.0, c["topk_idx"], c["topk_w"], c["counts"], c["offsets"], c["row_of"],
                           c["src_of"], c["Xp"], None, None, ws)
    torch.cuda.synchronize()
    assert torch.equal(c["row_of"], a["row_of"]) and bool(torch.isnan(c["P"]).all())
    # backward of the gate with the loss folded in
    dw = torch.randn(T, k, generator=torch.Generator().manual_seed(3)).to(dev)
    sep = torch.full((T, E), float("nan"), device=dev)
    fus = torch.full((T, E), float("nan"), device=dev)
    moe.moe_route_bwd(shape, lgd, a["topk_idx"], dw, sep)
    moe.moe_aux_loss_bwd(shape, lgd, a["counts"], alpha, 1.7, True, sep)
    moe.moe_route_aux_bwd(shape, lgd, a["topk_idx"], dw, a["counts"], alpha, 1.7, fus)
    torch.cuda.synchronize()
    ref = orc.route_bwd(lg.numpy(), ridx, dw.cpu().numpy(), gate, True) + orc.aux_loss_bwd(lg.numpy(), rc[0], k, alpha, gate, 1.7)
    assert scale_rel_err(fus.cpu(), ref) <= 1e-4 and scale_rel_err(sep.cpu(), ref) <= 1e-4
