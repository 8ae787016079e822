"""Static check of the generated code of the hand-pipelined backward kernels (no GPU needed).

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
