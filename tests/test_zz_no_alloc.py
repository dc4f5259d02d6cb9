"""moe_dispatch_static (the entry point that allocates nothing: its scratch is an array inside the
library) against moe_dispatch, through the C ABI, bit for bit; two calls in a row, the second on a
smaller input, so that stale scratch contents of the first call would show."""
import numpy as np
import pytest
import torch

import workloads as wl

pytestmark = pytest.mark.gpu


def _run_both(moe, T, E, k, d, seed):
    dev = "cuda:0"
    g = torch.Generator().manual_seed(seed)
    shape = moe.MoEShape(T, d, E, k, 64, "bf16")
    A = T * k
    logits = torch.randn(T, E, generator=g) + torch.log(torch.arange(1, E + 1, dtype=torch.float32) ** -1.2)
    idx = torch.topk(logits, k, dim=1).indices.to(torch.int32).to(dev)
    X = (torch.randn(T, d, generator=g) * 0.02).to(torch.bfloat16).to(dev)
    i32 = dict(dtype=torch.int32, device=dev)
    out = []
    for which in ("ws", "static"):
        # poisoned outputs: every element must be written by the call
        b = {"counts": torch.full((E,), -7, **i32), "offsets": torch.full((E + 1,), -7, **i32),
             "row_of": torch.full((A,), -7, **i32), "src_of": torch.full((A,), -7, **i32),
             "Xp": torch.full((A, d), float("nan"), dtype=torch.bfloat16, device=dev)}
        if which == "ws":
            ws = torch.empty(moe.moe_dispatch_workspace_bytes(shape), dtype=torch.uint8, device=dev)
            moe.moe_dispatch(shape, X, idx, b["counts"], b["offsets"], b["row_of"], b["src_of"], b["Xp"], ws)
        else:
            moe.moe_dispatch_static(shape, X, idx, b["counts"], b["offsets"], b["row_of"], b["src_of"], b["Xp"])
        torch.cuda.synchronize()
        out.append({n: t.cpu() for n, t in b.items()})
    ref, got = out
    for n in ("counts", "offsets", "row_of", "src_of"):
        assert np.array_equal(ref[n].numpy(), got[n].numpy()), n
    assert torch.equal(ref["Xp"].view(torch.int16), got["Xp"].view(torch.int16)), "Xp"
    # and what is unique about the result, independent of the other entry point
    counts = np.bincount(idx.cpu().numpy().reshape(-1), minlength=E)
    assert np.array_equal(got["counts"].numpy(), counts)
    assert np.array_equal(np.sort(got["row_of"].numpy()), np.arange(A))


def test_static_dispatch_matches_workspace_dispatch_twice():
    import paper_2502_02581_amd as moe

    # first call: several chunks of 256 assignments with a ragged last one; second call: smaller, on the
    # same (now dirty) scratch array
    _run_both(moe, T=1500, E=96, k=6, d=256, seed=1)
    _run_both(moe, T=333, E=40, k=3, d=128, seed=2)


def test_static_dispatch_empty_and_limit():
    import paper_2502_02581_amd as moe

    dev = "cuda:0"
    i32 = dict(dtype=torch.int32, device=dev)
    shape = moe.MoEShape(0, 64, 8, 2, 64, "bf16")
    counts, offsets = torch.full((8,), 5, **i32), torch.full((9,), 5, **i32)
    moe.moe_dispatch_static(shape, None, None, counts, offsets, None, None, None)
    torch.cuda.synchronize()
    assert int(counts.abs().sum()) == 0 and int(offsets.abs().sum()) == 0
    # beyond the built-in scratch: refused on the host, nothing launched
    big = moe.MoEShape(1 << 20, 64, 1024, 8, 64, "bf16")
    fake = torch.empty(16, dtype=torch.bfloat16, device=dev)
    fi = torch.empty(16, **i32)
    with pytest.raises(moe.MoEError, match="exceed the built-in scratch"):
        moe.moe_dispatch_static(big, fake, fi, fi, fi, fi, fi, fake)
