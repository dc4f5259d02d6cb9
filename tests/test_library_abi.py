"""CPU-side checks of the C-ABI library: it loads, exports every declared symbol, and rejects
bad arguments on the host before anything is launched (no GPU needed)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "moe_hip.h")


@pytest.fixture(scope="module")
def lib():
    import paper_2502_02581_amd as moe

    if not os.path.exists(moe.lib_path()):
        from paper_2502_02581_amd import build

        build.build(verbose=False)
    return moe.load_library()


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z_]+)\s*\(", text)))


def test_exports_every_declared_symbol(lib):
    names = declared_functions()
    assert {"moe_route", "moe_dispatch", "moe_expert_fwd", "moe_expert_bwd", "moe_combine"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in include/moe_hip.h but not exported"
    from paper_2502_02581_amd import binding

    assert sorted(binding.EXPORTS) == names


def test_abi_version_matches_header(lib):
    ver = int(re.search(r"#define MOE_ABI_VERSION (\d+)", open(HEADER).read()).group(1))
    assert lib.moe_abi_version() == ver


def test_host_side_validation(lib):
    import paper_2502_02581_amd as moe
    from paper_2502_02581_amd.binding import _CShape

    def shape(**kw):
        base = dict(T=16, d=64, E=8, k=2, d_ff=64, dtype=1, gate=0, renorm=1)
        base.update(kw)
        return _CShape(*[base[n] for n in ("T", "d", "E", "k", "d_ff", "dtype", "gate", "renorm")])

    fake = ctypes.c_void_p(4096)  # never dereferenced: every call below must fail before a launch
    cases = [
        (shape(d=60), -1, "multiples of 8"),
        (shape(k=9), -1, "bad shape"),
        (shape(E=2000), -1, "bad shape"),
        (shape(dtype=7), -3, "dtype"),
        (shape(gate=5), -3, "gate"),
        (shape(T=1 << 30, k=4, E=8), -1, "overflows"),
    ]
    for s, code, msg in cases:
        assert lib.moe_route(ctypes.byref(s), fake, fake, fake, None) == code
        assert msg in lib.moe_last_error().decode()
    s = shape()
    assert lib.moe_route(ctypes.byref(s), None, fake, fake, None) == -1
    assert "null" in lib.moe_last_error().decode()
    # misaligned tensor and short workspace
    assert lib.moe_combine(ctypes.byref(s), ctypes.c_void_p(4100), fake, fake, None, fake, None) == -1
    assert "aligned" in lib.moe_last_error().decode()
    assert lib.moe_dispatch(ctypes.byref(s), fake, fake, fake, fake, fake, fake, fake, fake, 16, None) == -2
    assert lib.moe_expert_fwd(ctypes.byref(s), 8, fake, 32, *([fake] * 9), 16, None) == -2
    assert lib.moe_expert_bwd(ctypes.byref(s), 8, fake, 32, *([fake] * 15), 16, None) == -2
    assert lib.moe_expert_fwd(ctypes.byref(s), 0, fake, 32, *([fake] * 9), 1 << 20, None) == -1
    lib.moe_aux_loss.argtypes = [ctypes.c_void_p] * 3 + [ctypes.c_float] + [ctypes.c_void_p] * 3 + [ctypes.c_size_t, ctypes.c_void_p]
    assert lib.moe_aux_loss(ctypes.byref(s), fake, fake, 0.001, fake, fake, fake, 16, None) == -2
    assert "workspace" in lib.moe_last_error().decode()
    # the dispatch without a workspace argument refuses what its built-in scratch cannot hold
    big = shape(T=1 << 20, k=8, E=1024)
    assert lib.moe_dispatch_static(ctypes.byref(big), fake, fake, fake, fake, fake, fake, fake, None) == -2
    assert "built-in scratch" in lib.moe_last_error().decode()
    # workspace queries are pure host arithmetic
    sh = moe.MoEShape(8192, 7168, 256, 8, 2048)
    assert moe.moe_dispatch_workspace_bytes(sh) >= 256 * 256 * 4
    grouped = moe.moe_expert_bwd_workspace_bytes(sh, 256, 65536, False)
    assert 2 * 65536 * 2048 * 2 <= grouped < 2 * 65536 * 2048 * 2 + (1 << 20)
    assert moe.moe_expert_bwd_workspace_bytes(sh, 1, 8192, True) >= 2 * 8192 * 2048 * 2


def test_missing_library_is_loud(monkeypatch, tmp_path):
    from paper_2502_02581_amd import binding

    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_HERE", str(tmp_path))
    with pytest.raises(binding.MoEError, match="no CPU or PyTorch fallback"):
        binding.load_library()
