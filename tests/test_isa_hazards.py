"""Static check of the generated gfx950 code (no GPU): loads issued from inline assembly are
invisible to the compiler's wait-count bookkeeping, so nothing may read or write their
destination registers before a wait that covers them, on any path.  The kernels guarantee that
by making those registers operands of the wait; this test compiles the kernels to assembly and
follows every path from every such load through the control-flow graph to confirm it.

The model: vector-memory operations of a wave complete in issue order, and `s_waitcnt vmcnt(N)`
returns when at most N of them are outstanding, so a load is complete once a wait with
N <= (vector-memory instructions issued after it) has been passed.  That rule is applied to the
compiler's own waits.  A wait written by hand (inside inline assembly) is taken to cover every
hand-issued load before it: its count is the kernel author's statement about the instructions
in between (the streaming loop waits with vmcnt(loads of the next tile), and both staging paths
issue exactly that many), which a path-insensitive pass over two complementary branches cannot
re-derive.  What this test does establish is that the registers stay untouched up to that wait."""
import collections
import os
import re
import subprocess

import pytest

from paper_2603_17435_amd import build as zs_build

VMEM = ("global_load", "global_store", "global_atomic", "scratch_load", "scratch_store", "buffer_load", "buffer_store",
        "flat_load", "flat_store", "flat_atomic")
SATURATED = 64  # vmcnt cannot name more


def registers(operand: str) -> set[int]:
    m = re.fullmatch(r"v\[(\d+):(\d+)\]", operand)
    if m:
        return set(range(int(m.group(1)), int(m.group(2)) + 1))
    m = re.fullmatch(r"v(\d+)", operand)
    return {int(m.group(1))} if m else set()


def kernels(asm: str):
    """(name, [(text, in_inline_asm)]) per kernel of the translation unit."""
    for km in re.finditer(r"^(_Z\w+):.*$", asm, re.M):
        end = asm.find(".end_amdhsa_kernel", km.end())
        nxt = re.search(r"^_Z\w+:.*$", asm[km.end():], re.M)
        if end < 0 or (nxt and km.end() + nxt.start() < end):
            continue
        ins, inline = [], False
        for line in asm[km.end():end].split("\n"):
            if "#ASMSTART" in line:
                inline = True
            if "#ASMEND" in line:
                inline = False
            text = line.split(";")[0].strip()
            if text and (not text.startswith(".") or re.match(r"\.LBB\d+_\d+:", text)):
                ins.append((text, inline))
        yield km.group(1), ins


def hazards(ins):
    label_at = {t[:-1]: i for i, (t, _) in enumerate(ins) if t.endswith(":")}
    n = len(ins)

    def successors(i):
        t = ins[i][0]
        if t.endswith(":"):
            return [i + 1]
        mn = t.split()[0]
        if mn == "s_endpgm":
            return []
        if mn == "s_branch":
            return [label_at[t.split()[1]]]
        if mn.startswith("s_cbranch"):
            return [label_at[t.split()[1]], i + 1]
        return [i + 1]

    state_in = [None] * n  # register -> fewest vector-memory instructions issued since its load, over all paths
    state_in[0] = {}
    work = collections.deque([0])
    found = {}
    while work:
        i = work.popleft()
        cur = dict(state_in[i])
        text, inline = ins[i]
        if not text.endswith(":"):
            parts = text.split(None, 1)
            mn = parts[0]
            ops = [o.strip() for o in parts[1].split(",")] if len(parts) > 1 else []
            if mn == "s_waitcnt":
                m = re.search(r"vmcnt\((\d+)\)", text)
                if m:
                    cur = {} if inline else {r: k for r, k in cur.items() if k < int(m.group(1))}
            else:
                asm_load = inline and mn.startswith("global_load") and "lds" not in mn
                touched = set().union(*(registers(o.split()[0]) for o in ops if o)) if ops else set()
                if not asm_load and touched & cur.keys():
                    found.setdefault(i, (text, sorted(touched & cur.keys())))
                if mn.startswith(VMEM):
                    cur = {r: min(k + 1, SATURATED) for r, k in cur.items()}
                if asm_load:
                    for r in registers(ops[0]):
                        cur[r] = 0
        for s in successors(i):
            if s >= n:
                continue
            old = state_in[s]
            new = dict(cur) if old is None else {r: min(cur.get(r, SATURATED), old.get(r, SATURATED)) for r in cur.keys() | old.keys()}
            if old is None or new != old:
                state_in[s] = new
                work.append(s)
    return found


@pytest.fixture(scope="module")
def kernel_asm(tmp_path_factory):
    out = tmp_path_factory.mktemp("isa") / "zs_kernels.s"
    src = os.path.join(zs_build.CSRC, "zs_kernels.hip")
    cmd = [zs_build.HIPCC, "-S", "--cuda-device-only", src, "-o", str(out)] + \
          [f for f in zs_build.COMMON if f != "-fPIC"] + zs_build.DEVICE
    subprocess.run(cmd, check=True, capture_output=True)
    return out.read_text()


def test_checker_sees_a_planted_hazard():
    """The checker on hand-made code: a register written while its load is in flight is reported,
    the same code with a covering wait is not, and a wait that leaves the load outstanding does not count."""
    def prog(wait):
        return [("s_nop 0", False), ("global_load_dwordx4 v[4:7], v1, s[2:3]", True), ("global_load_lds_dwordx4 v1, s[4:5]", True)] + \
               ([(wait, False)] if wait else []) + [("v_mov_b32_e32 v5, v0", False), ("s_endpgm", False)]
    assert hazards(prog(None))
    assert hazards(prog("s_waitcnt vmcnt(2)"))
    assert not hazards(prog("s_waitcnt vmcnt(1)"))
    assert not hazards(prog("s_waitcnt vmcnt(0)"))
    # a branch around the wait is a path without it
    branchy = [("global_load_dwordx4 v[4:7], v1, s[2:3]", True), ("s_cbranch_scc1 .LBB0_1", False), ("s_waitcnt vmcnt(0)", True),
               (".LBB0_1:", False), ("v_add_f32_e32 v0, v4, v0", False), ("s_endpgm", False)]
    assert hazards(branchy)


def test_no_register_of_a_hand_issued_load_is_touched_before_its_wait(kernel_asm):
    seen_loads = 0
    for name, ins in kernels(kernel_asm):
        seen_loads += sum(1 for t, inline in ins if inline and t.startswith("global_load") and "lds" not in t.split()[0])
        found = hazards(ins)
        assert not found, f"{name}: {list(found.values())[:4]}"
    assert seen_loads > 0  # the streaming kernels issue their activation fragments by hand
