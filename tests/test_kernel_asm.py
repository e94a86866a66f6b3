"""Host-side check of an invariant of the weight-gradient kernel that the compiler cannot see.

In its shared-planes path the loads are written as instructions and the waits are placed by hand
(`s_waitcnt vmcnt(n)` inside asm statements), so the compiler takes a load's destination register for a finished
value from the moment the load is issued.  Nothing may read or write such a register before the wait that covers
it -- in particular no register copy that the compiler inserts at a branch.  The kernel's control flow is shaped so
that the compiler has no reason to; this test compiles the file to assembly and walks every path from the first
of those loads, tracking which destinations are still in flight, to make sure it did not."""
import os
import re
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "paper_2501_15348_amd", "csrc", "kernels_dense.hip")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


@pytest.fixture(scope="module")
def assembly(tmp_path_factory):
    if not os.path.exists(HIPCC):
        pytest.skip("no hipcc")
    out = tmp_path_factory.mktemp("asm") / "kernels_dense.s"
    cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wno-unused-function", "-Xclang", "-target-feature",
           "-Xclang", "-packed-fp32-ops", "-I", os.path.join(ROOT, "include"), "-I", os.path.dirname(SRC), "--cuda-device-only",
           "-S", SRC, "-o", str(out)]
    subprocess.run(cmd, check=True, capture_output=True)
    return out.read_text().splitlines()


def _function(lines, mangled_part):
    start = next(k for k, l in enumerate(lines) if l.startswith("_Z") and mangled_part in l and l.rstrip().split(":")[0].endswith("E"))
    end = next(k for k in range(start, len(lines)) if lines[k].startswith(".Lfunc_end"))
    return lines[start + 1:end]


def _blocks(body):
    """Basic blocks keyed by label, in layout order; each a list of (text, in_asm)."""
    blocks, order, cur, in_asm = {"entry": []}, ["entry"], "entry", False
    for l in body:
        s = l.strip()
        if re.match(r"^\.LBB\d+_\d+:", s):
            cur = s.split(":")[0]
            blocks[cur] = []
            order.append(cur)
            continue
        if "ASMSTART" in s:
            in_asm = True
            continue
        if "ASMEND" in s:
            in_asm = False
            continue
        if not s or s.startswith(";") or s.startswith("."):
            continue
        blocks[cur].append((s, in_asm))
    return blocks, order


def _registers(text):
    regs = {int(r) for r in re.findall(r"\bv(\d+)\b", text)}
    for a, b in re.findall(r"v\[(\d+):(\d+)\]", text):
        regs |= set(range(int(a), int(b) + 1))
    return regs


def _walk(blocks, order):
    """Every path from the block with the first hand-written load; returns (violations, hand-written loads seen)."""
    first = next(b for b in order if any(a and t.startswith("global_load") for t, a in blocks[b]))
    nxt = {b: order[i + 1] if i + 1 < len(order) else None for i, b in enumerate(order)}
    seen, todo, violations, loads = set(), [(first, ())], [], 0
    while todo:
        name, state = todo.pop()
        if name is None or (name, state) in seen:
            continue
        seen.add((name, state))
        inflight, ended = list(state), False
        for text, in_asm in blocks[name]:
            if in_asm and text.startswith("global_load"):
                inflight.append(int(re.match(r"global_load_dword v(\d+)", text).group(1)))
                loads += 1
                continue
            if in_asm and text.startswith("s_waitcnt"):
                n = int(re.search(r"vmcnt\((\d+)\)", text).group(1))
                inflight = inflight[len(inflight) - n:] if n else []
                continue
            hit = _registers(text) & set(inflight)
            if hit and not text.startswith("s_"):
                violations.append((name, text, sorted(hit)))
            if text.startswith("s_endpgm"):
                ended = True
                break
            m = re.match(r"s_(c?branch\w*)\s+(\.LBB\d+_\d+)", text)
            if m:
                todo.append((m.group(2), tuple(inflight)))
                if m.group(1) == "branch":
                    ended = True
                    break
        if not ended:
            todo.append((nxt[name], tuple(inflight)))
        assert len(seen) < 200000, "path walk did not converge"
    return violations, loads


@pytest.mark.parametrize("variant", ["ILb0ELb1ELb1E", "ILb1ELb1ELb1E"])  # <HAS_RS, SPLIT = true, WIDE = true>
def test_nothing_touches_a_register_with_a_load_in_flight(assembly, variant):
    body = _function(assembly, "gemm_reduce_kernel" + variant)
    blocks, order = _blocks(body)
    violations, loads = _walk(blocks, order)
    assert loads >= 5 * 16, "the hand-written loads were not found: has the kernel changed?"
    assert not violations, violations[:5]


def test_the_walk_finds_a_planted_copy(assembly):
    """The checker itself: a copy of an in-flight destination planted after the first hand-written load is reported."""
    body = list(_function(assembly, "gemm_reduce_kernelILb0ELb1ELb1E"))
    k = next(i for i, l in enumerate(body) if l.strip().startswith("global_load_dword") and "ASMSTART" in body[i - 1])
    reg = re.match(r"global_load_dword (v\d+)", body[k].strip()).group(1)
    body.insert(k + 2, f"\tv_mov_b32_e32 v255, {reg}")
    violations, _ = _walk(*_blocks(body))
    assert any(reg[1:] == str(h) for _, _, hit in violations for h in hit)


def _loop_blocks(blocks, order):
    """Labels of the blocks between the first block that holds matrix instructions and the last block that branches
    back to it or before it: the kernel's loops over chunks."""
    index = {b: k for k, b in enumerate(order)}
    first = next(k for k, b in enumerate(order) if any(t.startswith("v_mfma") for t, _ in blocks[b]))
    last = first
    for k, b in enumerate(order):
        for t, _ in blocks[b]:
            m = re.match(r"s_c?branch\w*\s+(\.LBB\d+_\d+)", t)
            if m and first <= index[m.group(1)] <= k:
                last = max(last, k)
    return order[first:last + 1]


def test_packed_lstm_cell_keeps_its_loads_in_flight_and_its_epilogue_short(assembly):
    """Two properties of the compiled packed LSTM step that the source cannot state.  (1) Inside the steady loop no
    wait drains the ring of row loads: the epilogue issues no loads of its own (the previous cell state arrives as a
    chunk), so every vmcnt wait there leaves the newest chunks in flight.  (2) The exchange between the two lanes of a
    hidden unit is one select per value: once it had been compiled into an element at a selected index, a chain of 15
    selects per value (1860 selects in the loop instead of 275)."""
    body = _function(assembly, "rnn_fused_resident_kernelILb1ELi1ELi8ELb1ELb1E")
    blocks, order = _blocks(body)
    loop = _loop_blocks(blocks, order)
    chunk_blocks = [b for b in loop if sum(t.startswith("v_mfma") for t, _ in blocks[b]) >= 24]
    assert len(chunk_blocks) >= 4, "the unrolled chunk steps were not found: has the kernel changed?"
    steady = loop[:loop.index(chunk_blocks[3]) + 1]  # the first loop: one step per ring buffer, loads unconditional
    waits = [int(n) for b in steady for t, _ in blocks[b] for n in re.findall(r"vmcnt\((\d+)\)", t)]
    assert waits and min(waits) >= 10, sorted(set(waits))
    selects = sum(t.startswith("v_cndmask") for b in steady for t, _ in blocks[b])
    assert selects <= 600, selects
