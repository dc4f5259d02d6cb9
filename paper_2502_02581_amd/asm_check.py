"""Checks of the device assembly that hipcc emits for the GEMM kernels (run by build.py).

The tile loads of the LDS-DMA cores are inline assembly, which the compiler's hazard recogniser does
not look into.  Two things it would otherwise guarantee are therefore checked on the emitted code:

  * a scalar register of the buffer descriptor that such a load reads must not have been written by a
    vector instruction (v_readfirstlane, v_readlane of a spilled scalar, a compare or carry-out) in
    the five wait states before the load, along any path of the control flow that reaches the load:
    loop back edges and both arms of a branch are followed (the M0 write in front of the load is a
    scalar instruction and has its own wait state inside the inline assembly);
  * no GEMM kernel keeps anything in scratch memory: accumulator tiles that end up there (an
    epilogue too large to unroll did that once) cost a factor of four and show up nowhere else;
  * no packed fp32 arithmetic (v_pk_add_f32, v_pk_mul_f32, v_pk_fma_f32): the build switches the
    feature off (`-packed-fp32-ops`), and this makes sure the switch is still in the flags.

`check(path)` returns a list of findings (empty: fine); `python -m paper_2502_02581_amd.asm_check file.s`
prints them.
"""
from __future__ import annotations

import re
import sys
from typing import List, Set

WAIT_STATES = 5
# vector instructions whose first or second operand may be a scalar destination
_SCALAR_WRITERS = ("v_readfirstlane", "v_readlane", "v_cmp", "v_add_co", "v_sub_co", "v_subrev_co", "v_addc_co",
                   "v_subb_co", "v_subbrev_co", "v_div_scale", "v_mad_u64_u32", "v_mad_i64_i32")


def _sregs(tok: str) -> Set[int]:
    tok = tok.strip()
    m = re.match(r"s\[(\d+):(\d+)\]$", tok)
    if m:
        return set(range(int(m.group(1)), int(m.group(2)) + 1))
    m = re.match(r"s(\d+)$", tok)
    if m:
        return {int(m.group(1))}
    return set()


_LABEL = re.compile(r"^([.\w$]+):")


def _instructions(lines: List[str]):
    for i, raw in enumerate(lines):
        t = raw.strip()
        if not t or t.startswith(";") or t.startswith(".") or t.endswith(":") or t.startswith("//"):
            continue
        yield i + 1, t


def _control_flow(lines: List[str]):
    """The instructions of a file as (line number, text) and, for each, the indices of the instructions
    that may execute right before it: the one above (unless that one never falls through) and every
    branch whose target label stands in front of it -- loop back edges and the far arm of an `if`
    included."""
    ins, label_at = [], {}
    pending = []
    for i, raw in enumerate(lines):
        t = raw.strip()
        m = _LABEL.match(t)
        if m and not t.startswith("//"):
            pending.append(m.group(1))
            continue
        if not t or t.startswith(";") or t.startswith(".") or t.startswith("//"):
            continue
        for name in pending:
            label_at[name] = len(ins)
        pending = []
        ins.append((i + 1, t))
    preds = [set() for _ in ins]
    for k, (_, t) in enumerate(ins):
        op = t.split()[0]
        falls = op not in ("s_branch", "s_endpgm", "s_setpc_b64", "s_swappc_b64")
        if falls and k + 1 < len(ins):
            preds[k + 1].add(k)
        if op == "s_branch" or op.startswith("s_cbranch"):
            target = t.split()[-1]
            if target in label_at and label_at[target] < len(ins):
                preds[label_at[target]].add(k)
    return ins, preds


def _scalar_dests(t: str) -> Set[int]:
    parts = t.split(None, 1)
    if len(parts) < 2 or not parts[0].startswith(_SCALAR_WRITERS):
        return set()
    ops = [o.strip() for o in parts[1].split(",")]
    out: Set[int] = set()
    for o in ops[:2]:
        out |= _sregs(o)
    return out


def check_descriptor_hazards(lines: List[str]) -> List[str]:
    """Walks backwards from every LDS-DMA load along every path of the control flow (not the order of the
    file: a writer at the tail of a loop, or in the other arm of a branch, precedes the load in
    execution just as well) until WAIT_STATES wait states have passed."""
    ins, preds = _control_flow(lines)
    findings = []
    for k, (ln, t) in enumerate(ins):
        if not (t.startswith("buffer_load") and t.endswith(" lds")):
            continue
        read = set()
        for o in t.split(None, 1)[1].split(","):
            read |= _sregs(o.split()[0] if o.strip() else "")
        best = {}                      # instruction -> fewest wait states at which it was reached
        stack = [(j, 0) for j in preds[k]]
        seen_hits = set()
        while stack:
            j, ws = stack.pop()
            if ws >= WAIT_STATES or best.get(j, WAIT_STATES) <= ws:
                continue
            best[j] = ws
            u = ins[j][1]
            hit = _scalar_dests(u) & read
            if hit and j not in seen_hits:
                seen_hits.add(j)
                findings.append(f"line {ln}: `{t}` reads s{sorted(hit)} written by `{u}` (line {ins[j][0]}) "
                                f"{ws} wait states earlier")
            op = u.split()[0]
            nxt = ws + (int(u.split()[1]) + 1 if op == "s_nop" else 1)
            stack.extend((q, nxt) for q in preds[j])
    return findings


def check_no_scratch(lines: List[str], name_part: str = "gemm_kernel") -> List[str]:
    findings = []
    kernel = None
    for raw in lines:
        t = raw.strip()
        m = re.match(r"^(_Z\w+):", t)
        if m:
            kernel = m.group(1)
        m = re.match(r"^; ScratchSize: (\d+)", t)
        if m and kernel and name_part in kernel and int(m.group(1)) != 0:
            findings.append(f"{kernel}: {m.group(1)} bytes of scratch memory per lane")
    return findings


def check_no_packed_fp32(lines: List[str]) -> List[str]:
    findings = []
    for ln, t in _instructions(lines):
        if t.startswith(("v_pk_add_f32", "v_pk_mul_f32", "v_pk_fma_f32")):
            findings.append(f"line {ln}: packed fp32 instruction `{t}`")
            if len(findings) >= 5:
                break
    return findings


def check(path: str) -> List[str]:
    with open(path) as f:
        lines = f.read().split("\n")
    return check_descriptor_hazards(lines) + check_no_scratch(lines) + check_no_packed_fp32(lines)


if __name__ == "__main__":
    bad = check(sys.argv[1])
    print("\n".join(bad) if bad else "no findings")
    sys.exit(1 if bad else 0)
