"""Static checks of the generated code of kernels with inline-assembly LDS reads (no GPU needed).

The operand reads of k_bwd_dkv2 and k_bwd_dq2 are inline-assembly LDS reads whose completion the
compiler does not track: the kernels wait for them with explicit lgkmcnt counts.  That is only
sound if, in the generated code, (a) a pipelined iteration is one straight-line block (a branch
inside it could make the register allocator copy a register that is still being written), and
(b) no instruction touches the destination of a read that may still be pending under the in-order
return of LDS reads.  This test compiles the source to assembly and checks both, so that a
compiler or source change that breaks the scheme is found on the CPU and not as wrong gradients.
"""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "paper_2602_07529_amd", "csrc", "prefill_bwd.hip")
HIPCC = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"

# kernel -> LDS reads of its pipelined blocks (without masks, with masks)
#   k_bwd_dkv2: 32 row operands + 32 transposed operands (two reads each) + 8 groups of row data (2 or 3 reads)
#   k_bwd_dq2:  32 row operands + 16 transposed operands (two reads each) (+ 8 reads of node ids)
EXPECTED = {"k_bwd_dkv2": [112, 120], "k_bwd_dq2": [64, 72]}


def _regs(text):
    out = set()
    for m in re.finditer(r"\bv\[(\d+):(\d+)\]|\bv(\d+)\b", text):
        if m.group(1):
            out |= set(range(int(m.group(1)), int(m.group(2)) + 1))
        else:
            out.add(int(m.group(3)))
    return out


def _blocks(lines):
    """Straight-line runs of instructions: split at labels and after branches."""
    cur = []
    for raw in lines:
        l = raw.split(";")[0].strip()
        if not l:
            continue
        if re.match(r"^\.?[A-Za-z_][\w.$]*:$", l):
            if cur:
                yield cur
            cur = []
            continue
        if l.startswith("."):
            continue
        cur.append(l)
        if l.startswith(("s_cbranch", "s_branch", "s_endpgm", "s_setpc")):
            yield cur
            cur = []
    if cur:
        yield cur


def _check_block(block):
    """Returns (reads, conflicts, pending at the end) under the in-order lgkmcnt model."""
    pending, conflicts, reads = [], [], 0
    for l in block:
        op = l.split()[0]
        args = l[len(op):]
        if op.startswith("ds_read"):
            parts = args.split(",")
            dst, src = _regs(parts[0]), _regs(",".join(parts[1:]))
            conflicts += [l for d in pending if d & (dst | src)]
            pending.append(dst)
            reads += 1
        elif op == "s_waitcnt":
            m = re.search(r"lgkmcnt\((\d+)\)", l)
            if m and int(m.group(1)) < len(pending):
                n = int(m.group(1))
                pending = pending[len(pending) - n:] if n else []
        else:
            touched = _regs(args)
            conflicts += [l for d in pending if d & touched]
    return reads, conflicts, len(pending)


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="no hipcc")
def test_pipelined_backward_blocks_keep_pending_reads_untouched(tmp_path):
    asm = tmp_path / "prefill_bwd.s"
    cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fno-gpu-rdc", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
           "-I" + os.path.join(ROOT, "include"), "-I" + os.path.dirname(SRC), "-S", "--cuda-device-only", "-o", str(asm), SRC]
    subprocess.run(cmd, check=True, capture_output=True, timeout=900)
    text = asm.read_text().split("\n")
    for kernel, expected in EXPECTED.items():
        start = next(i for i, l in enumerate(text) if re.match(r"^_Z\w*%s\w*:" % kernel, l))
        end = next(i for i in range(start, len(text)) if "s_endpgm" in text[i])
        found = []
        for block in _blocks(text[start + 1:end + 1]):
            reads, conflicts, left = _check_block(block)
            # a pipelined block holds a whole iteration (64 or 48 MFMAs); the blocks of the general walks, whose
            # reads the compiler tracks itself, hold 16 at most
            if sum(1 for l in block if l.startswith("v_mfma")) >= 40:
                assert not conflicts, "%s: an instruction touches a register with a read in flight: %s" % (kernel, conflicts[:3])
                assert left == 0, "%s: a pipelined block ends with %d reads in flight (a branch inside it?)" % (kernel, left)
                found.append(reads)
            else:
                # elsewhere an inline read waits for itself, and the compiler waits for its own reads
                assert not conflicts, "%s: %s" % (kernel, conflicts[:3])
        assert sorted(found) == sorted(expected), "%s: pipelined blocks with %s reads, expected %s" % (kernel, found, expected)


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


def _run_block(insts, inherited):
    """Registers with a read possibly in flight at the end of the block, and the instructions that touch such
    a register.  `inherited`: registers possibly in flight at the entry (all older than this block's reads, so
    a wait that leaves at most as many reads as the block has issued itself covers them)."""
    inherited, local, issued, conflicts = set(inherited), [], 0, []
    for l in insts:
        op = l.split()[0]
        args = l[len(op):]
        if op.startswith("ds_read"):
            parts = args.split(",")
            dst, src = _regs(parts[0]), _regs(",".join(parts[1:]))
            if (dst | src) & inherited or any(d & (dst | src) for d in local):
                conflicts.append(l)
            local.append(dst)
            issued += 1
        elif op == "s_waitcnt":
            m = re.search(r"lgkmcnt\((\d+)\)", l)
            if m:
                n = int(m.group(1))
                if n <= issued:
                    inherited = set()
                if n < len(local):
                    local = local[len(local) - n:] if n else []
        else:
            t = _regs(args)
            if t & inherited or any(d & t for d in local):
                conflicts.append(l)
    out = set(inherited)
    for d in local:
        out |= d
    return out, conflicts


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="no hipcc")
def test_wide_decode_kernel_reads_are_waited_for_on_every_path(tmp_path):
    """k_decode_wide has branches between its inline reads' blocks (waves without a block in the
    last round, the skewed half of the waves): the registers that may have a read in flight are
    propagated over the control-flow graph (conservatively: the union over the predecessors), and
    no instruction may touch one."""
    src = os.path.join(os.path.dirname(SRC), "decode.hip")
    asm = tmp_path / "decode.s"
    cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fno-gpu-rdc", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
           "-I" + os.path.join(ROOT, "include"), "-I" + os.path.dirname(SRC), "-S", "--cuda-device-only", "-o", str(asm), src]
    subprocess.run(cmd, check=True, capture_output=True, timeout=900)
    text = asm.read_text().split("\n")
    starts = [i for i, l in enumerate(text) if re.match(r"^_Z\w*k_decode_wide\w*:", l)]
    assert len(starts) == 2  # head dimensions 128 and 64
    for st in starts:
        end = next(i for i in range(st, len(text)) if text[i].startswith(".Lfunc_end"))
        blocks = _cfg(text[st + 1:end + 1])
        entry = [set() for _ in blocks]
        changed = True
        while changed:
            changed = False
            for i, b in enumerate(blocks):
                out, _ = _run_block(b["insts"], entry[i])
                for nxt in b["succ"]:
                    if not out <= entry[nxt]:
                        entry[nxt] |= out
                        changed = True
        assert sum(1 for b in blocks for l in b["insts"] if l.startswith("ds_read_b128")) >= 12
        for i, b in enumerate(blocks):
            _, conflicts = _run_block(b["insts"], entry[i])
            assert not conflicts, conflicts[:3]


def test_the_checker_finds_a_planted_mistake():
    good = ["ds_read_b128 v[4:7], v1 offset:16", "ds_read_b128 v[8:11], v1 offset:32", "s_waitcnt lgkmcnt(1)",
            "v_mfma_f32_32x32x16_bf16 a[0:15], v[4:7], v[20:23], a[0:15]", "s_waitcnt lgkmcnt(0)",
            "v_mfma_f32_32x32x16_bf16 a[0:15], v[8:11], v[20:23], a[0:15]"]
    assert _check_block(good) == (2, [], 0)
    early = list(good)
    early[2] = "s_waitcnt lgkmcnt(2)"  # the first product would start before its operand has arrived
    assert _check_block(early)[1]
    copied = good[:1] + ["v_mov_b32_e32 v30, v5"] + good[1:]  # a copy of a register that is still being written
    assert _check_block(copied)[1]
    cut = good[:2]  # a block that ends (a branch) with reads in flight
    assert _check_block(cut)[2] == 2
    # over a branch: the read of the first block is still in flight when the second one copies its register
    two = ["ds_read_b128 v[4:7], v1", "s_cbranch_scc1 .LBB0_2", ".LBB0_1:", "s_waitcnt lgkmcnt(0)", ".LBB0_2:",
           "v_mov_b32_e32 v30, v5", "s_endpgm"]
    blocks = _cfg(two)
    out0, _ = _run_block(blocks[0]["insts"], set())
    assert out0 == {4, 5, 6, 7} and _run_block(blocks[2]["insts"], out0)[1]
    assert not _run_block(blocks[1]["insts"] + blocks[2]["insts"], out0)[1]   # after the wait it is fine
