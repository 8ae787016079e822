"""Static checks of the generated code of the kernels with inline-assembly LDS reads (no GPU needed).

The operand reads of the prefill, backward and wide-decode kernels are inline-assembly LDS reads
whose completion the compiler does not track: the kernels wait for them with explicit lgkmcnt
counts.  As far as the compiler knows such a read has written its register at once, so it may
copy the register, or (once the value is dead) reuse it for something else, while the read is
still in flight.  This test compiles the sources to assembly and checks, over the control-flow
graph of every kernel, that no instruction touches a register whose read may be pending under the
in-order return of LDS operations -- so that a compiler or source change that breaks the scheme is
found on the CPU and not as wrong numbers now and then.  For the two pipelined backward kernels it
also checks that an iteration is one straight-line block.
"""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2602_07529_amd", "csrc")
HIPCC = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
CAP = 24  # reads remembered per path (the hardware counter holds 15)

# pipelined blocks of the backward kernels (one without masks, one with): LDS reads of each
#   k_bwd_dkv2: 32 row operands + 32 transposed operands (two reads each) + 8 groups of row data (2 reads)
#   k_bwd_dq2:  32 row operands + 16 transposed operands (two reads each)
PIPELINED = {"k_bwd_dkv2": [112, 112], "k_bwd_dq2": [64, 64]}


def _regs(text):
    out = set()
    for m in re.finditer(r"\bv\[(\d+):(\d+)\]|\bv(\d+)\b", text):
        if m.group(1):
            out |= set(range(int(m.group(1)), int(m.group(2)) + 1))
        else:
            out.add(int(m.group(3)))
    return out


def _cfg(lines):
    """Basic blocks with successors, from labels and branches."""
    blocks, cur = [], {"labels": [], "insts": []}
    for raw in lines:
        l = raw.split(";")[0].strip()
        if not l:
            continue
        m = re.match(r"^(\.?[A-Za-z_][\w.$]*):$", l)
        if m:
            if cur["insts"]:
                blocks.append(cur)
                cur = {"labels": [], "insts": []}
            cur["labels"].append(m.group(1))
            continue
        if l.startswith("."):
            continue
        cur["insts"].append(l)
        if l.startswith(("s_cbranch", "s_branch", "s_endpgm", "s_setpc")):
            blocks.append(cur)
            cur = {"labels": [], "insts": []}
    if cur["insts"]:
        blocks.append(cur)
    where = {x: i for i, b in enumerate(blocks) for x in b["labels"]}
    for i, b in enumerate(blocks):
        last = b["insts"][-1]
        if last.startswith(("s_endpgm", "s_setpc")):
            b["succ"] = []
        elif last.startswith("s_branch"):
            b["succ"] = [where[last.split()[1]]]
        elif last.startswith("s_cbranch"):
            b["succ"] = [where[last.split()[1]]] + ([i + 1] if i + 1 < len(blocks) else [])
        else:
            b["succ"] = [i + 1] if i + 1 < len(blocks) else []
    return blocks


def _run(insts, pending):
    """pending: destination registers of the LDS operations possibly in flight, oldest first (an empty set for
    an LDS operation without a destination).  LDS operations return in order, so `s_waitcnt lgkmcnt(n)` leaves
    the newest n.  Scalar loads share the counter but may return early: they are left out, which only makes
    the waits look weaker.  Returns the list at the end and the instructions that touch a pending register."""
    pending, conflicts = list(pending), []
    for l in insts:
        op = l.split()[0]
        args = l[len(op):]
        if op.startswith("ds_read"):
            parts = args.split(",")
            dst, src = _regs(parts[0]), _regs(",".join(parts[1:]))
            if any(d & (dst | src) for d in pending):
                conflicts.append(l)
            pending = (pending + [frozenset(dst)])[-CAP:]
        elif op.startswith("ds_"):
            if any(d & _regs(args) for d in pending):
                conflicts.append(l)
            pending = (pending + [frozenset()])[-CAP:]
        elif op == "s_waitcnt":
            m = re.search(r"lgkmcnt\((\d+)\)", l)
            if m and int(m.group(1)) < len(pending):
                n = int(m.group(1))
                pending = pending[len(pending) - n:] if n else []
        elif any(d & _regs(args) for d in pending):
            conflicts.append(l)
    return pending, conflicts


def _merge(a, b):
    """Where paths meet: the lists aligned at their newest entry (waits cut from the oldest end), entry by entry
    the union."""
    n = max(len(a), len(b))
    at = lambda x, k: x[len(x) - n + k] if len(x) - n + k >= 0 else frozenset()
    return [at(a, k) | at(b, k) for k in range(n)][-CAP:]


def _conflicts_of_kernel(lines):
    blocks = _cfg(lines)
    entry = [[] for _ in blocks]
    changed, rounds = True, 0
    while changed:
        changed, rounds = False, rounds + 1
        assert rounds < 500, "no fixed point"
        for i, b in enumerate(blocks):
            out, _ = _run(b["insts"], entry[i])
            for s in b["succ"]:
                m = _merge(entry[s], out)
                if m != entry[s]:
                    entry[s], changed = m, True
    bad = []
    for i, b in enumerate(blocks):
        bad += _run(b["insts"], entry[i])[1]
    return blocks, bad


def _assembly(name, tmp_path):
    asm = tmp_path / (name + ".s")
    cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fno-gpu-rdc", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
           "-I" + os.path.join(ROOT, "include"), "-I" + CSRC, "-S", "--cuda-device-only", "-o", str(asm),
           os.path.join(CSRC, name + ".hip")]
    subprocess.run(cmd, check=True, capture_output=True, timeout=900)
    return asm.read_text().split("\n")


def _kernels(text, pattern):
    for st in [i for i, l in enumerate(text) if re.match(r"^_Z\w*%s\w*:" % pattern, l)]:
        end = next(i for i in range(st, len(text)) if text[i].startswith(".Lfunc_end"))
        yield text[st].split(":")[0], text[st + 1:end + 1]


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="no hipcc")
@pytest.mark.parametrize("source,pattern,n_kernels", [("prefill_bf16", "k_prefill_bf16", 6), ("prefill_bwd", "k_bwd_d", 17),
                                                      ("decode", "k_decode", 10)])
def test_no_instruction_touches_a_register_with_a_read_in_flight(tmp_path, source, pattern, n_kernels):
    text = _assembly(source, tmp_path)
    seen = 0
    for name, lines in _kernels(text, pattern):
        blocks, bad = _conflicts_of_kernel(lines)
        assert not bad, "%s: %s" % (name, bad[:3])
        seen += 1
        pipelined = [k for k in PIPELINED if k in name]
        if pipelined:
            # an iteration (64 or 48 MFMAs) is one straight-line block that starts and ends with nothing in flight
            found = []
            for b in blocks:
                if sum(1 for l in b["insts"] if l.startswith("v_mfma")) >= 40:
                    left, _ = _run(b["insts"], [])
                    assert not left, "%s: a pipelined block ends with %d reads in flight (a branch inside it?)" % (name, len(left))
                    found.append(sum(1 for l in b["insts"] if l.startswith("ds_read")))
            assert sorted(found) == PIPELINED[pipelined[0]], "%s: pipelined blocks with %s reads" % (name, found)
    assert seen == n_kernels


def test_the_checker_finds_planted_mistakes():
    good = ["ds_read_b128 v[4:7], v1 offset:16", "ds_read_b128 v[8:11], v1 offset:32", "s_waitcnt lgkmcnt(1)",
            "v_mfma_f32_32x32x16_bf16 a[0:15], v[4:7], v[20:23], a[0:15]", "s_waitcnt lgkmcnt(0)",
            "v_mfma_f32_32x32x16_bf16 a[0:15], v[8:11], v[20:23], a[0:15]"]
    assert _run(good, []) == ([], [])
    early = list(good)
    early[2] = "s_waitcnt lgkmcnt(2)"  # the first product would start before its operand has arrived
    assert _run(early, [])[1]
    copied = good[:1] + ["v_mov_b32_e32 v30, v5"] + good[1:]  # a copy of a register that is still being written
    assert _run(copied, [])[1]
    reused = good[:2] + ["v_max_f32_e32 v9, v40, v41"]  # a dead operand's register taken for a temporary too early
    assert _run(reused, [])[1]
    assert len(_run(good[:2], [])[0]) == 2  # a block that ends (a branch) with reads in flight
    # over a branch: on one path the read of the first block is still in flight when the last block copies its register
    two = ["ds_read_b128 v[4:7], v1", "s_cbranch_scc1 .LBB0_2", ".LBB0_1:", "s_waitcnt lgkmcnt(0)", ".LBB0_2:",
           "v_mov_b32_e32 v30, v5", "s_endpgm"]
    assert _conflicts_of_kernel(two)[1] == ["v_mov_b32_e32 v30, v5"]
    two[1] = "s_nop 0"  # without the branch every path passes the wait
    assert not _conflicts_of_kernel(two)[1]
    # a scalar load between a read and its wait does not count as a newer entry of the queue
    assert _run(["ds_read_b128 v[4:7], v1", "s_load_dword s4, s[0:1], 0x0", "s_waitcnt lgkmcnt(1)", "v_mov_b32_e32 v30, v5"], [])[1]
