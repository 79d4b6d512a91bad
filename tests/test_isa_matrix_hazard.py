"""Static check of the compiled decode kernels (no GPU needed): two matrix instructions of different depth on one
accumulator are kept far enough apart.

A half-depth step (v_mfma_f32_16x16x16_f16) issued right behind a full-depth step (v_mfma_f32_16x16x32_f16) that writes
its C operand read the accumulator too early on the hardware and lost the first step's contribution; the compiler adds
no wait states for that pair.  The kernels therefore put 20 wait states between the two groups (xdl_wait_states in
csrc/rinr_xdl.hip.h), pinned through data dependencies.  This test compiles the kernels to gfx950 assembly and measures,
for every matrix instruction whose C operand was last written by a matrix instruction of another opcode, the wait states
between the two (one per instruction issued in between, n + 1 for `s_nop n`): a later compiler or a change of the
kernels that moves them together again fails here, on the CPU, before any GPU run.
"""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "paper_2306_16699_amd", "csrc", "rinr_api.hip")
FIT_SRC = os.path.join(ROOT, "paper_2306_16699_amd", "csrc", "rinr_fit.hip")
MIN_WAIT_STATES = 20

MFMA = re.compile(r"^\s+(v_mfma_\w+)\s+([av])\[(\d+):(\d+)\],\s*\S+,\s*\S+,\s*(?:([av])\[(\d+):(\d+)\]|\S+)")
VWRITE = re.compile(r"^\s+(?:v_|ds_read|ds_add_rtn|global_load|buffer_load|flat_load)\S*\s+([av])(?:\[(\d+):(\d+)\]|(\d+))")
NOP = re.compile(r"^\s+s_nop\s+(\d+)")


def scan_kernel(lines):
    """Smallest distance in wait states between a matrix instruction and the matrix instruction of another opcode that
    last wrote its C operand; None if the kernel has no such pair.  Straight-line scan: a register written by any
    other vector instruction in between no longer belongs to the matrix instruction."""
    writer = {}           # (bank, register) -> (wait states so far, opcode)
    states = 0
    worst = None
    for ln in lines:
        m = NOP.match(ln)
        states += int(m.group(1)) + 1 if m else 1
        m = MFMA.match(ln)
        if not m:
            w = VWRITE.match(ln)
            if w and not re.match(r"^\s+v_cmpx?_", ln):
                lo, hi = (int(w.group(2)), int(w.group(3))) if w.group(2) else (int(w.group(4)), int(w.group(4)))
                for r in range(lo, hi + 1):
                    writer.pop((w.group(1), r), None)
            continue
        op, dbank, d0, d1, cbank, c0, c1 = m.groups()
        if cbank is not None:
            for r in range(int(c0), int(c1) + 1):
                prev = writer.get((cbank, r))
                if prev and prev[1] != op:
                    dist = states - prev[0]
                    if worst is None or dist < worst[0]:
                        worst = (dist, prev[1], op)
        for r in range(int(d0), int(d1) + 1):
            writer[(dbank, r)] = (states, op)
    return worst


def kernels_of(asm_text):
    name, body = None, []
    for ln in asm_text.splitlines():
        m = re.match(r"^(_Z\w+):", ln)
        if m:
            if name:
                yield name, body
            name, body = m.group(1), []
        elif name is not None:
            s = ln.strip()
            if s.startswith(".Lfunc_end"):
                yield name, body
                name, body = None, []
            elif s and not s.startswith(";") and not s.startswith(".") and not s.endswith(":"):
                body.append(ln)
    if name:
        yield name, body


def test_scanner_sees_a_close_pair_and_a_separated_one():
    close = ["\tv_mfma_f32_16x16x32_f16 v[0:3], v[8:11], v[12:15], v[0:3]",
             "\tv_sin_f32_e32 v20, v21",
             "\tv_mfma_f32_16x16x16_f16 v[0:3], v[16:17], v[18:19], v[0:3]"]
    assert scan_kernel(close)[0] == 2
    apart = close[:1] + ["\ts_nop 15", "\ts_nop 3"] + close[1:]
    assert scan_kernel(apart)[0] == 22
    same = [close[0], close[0]]
    assert scan_kernel(same) is None                      # one opcode: the case the hardware interlocks
    rewritten = [close[0], "\tds_read_b128 v[0:3], v40", close[2]]
    assert scan_kernel(rewritten) is None                 # the accumulator was reloaded: no dependency on the first


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="hipcc not found")
def test_mixed_depth_matrix_steps_stay_apart(tmp_path):
    out = tmp_path / "rinr_api.s"
    cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wno-unused-command-line-argument", "--cuda-device-only", "-S", "-o", str(out), SRC]
    subprocess.run(cmd, check=True, stdout=subprocess.DEVNULL, stderr=subprocess.PIPE)
    text = out.read_text()
    n_kernels = n_pairs = 0
    bad = []
    for name, body in kernels_of(text):
        if "decode" not in name:
            continue
        n_kernels += 1
        worst = scan_kernel(body)
        if worst is None:
            continue
        n_pairs += 1
        if worst[0] < MIN_WAIT_STATES:
            bad.append((name, worst))
    assert n_kernels >= 20 and n_pairs >= 10, (n_kernels, n_pairs)   # the scan found the kernels and the mixed-depth pairs
    assert not bad, bad


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="hipcc not found")
def test_fit_kernels_use_one_matrix_opcode_per_accumulator(tmp_path):
    """The fit kernels avoid the case altogether: each family uses a single matrix instruction (the split-precision ones
    pad an odd last tile with zeros rather than take a half-depth step)."""
    out = tmp_path / "rinr_fit.s"
    cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wno-unused-command-line-argument", "--cuda-device-only", "-S", "-o", str(out), FIT_SRC]
    subprocess.run(cmd, check=True, stdout=subprocess.DEVNULL, stderr=subprocess.PIPE)
    seen = 0
    for name, body in kernels_of(out.read_text()):
        if "step_kernel" not in name:
            continue
        ops = {m.group(1) for m in map(MFMA.match, body) if m}
        assert len(ops) == 1, (name, ops)
        assert scan_kernel(body) is None
        seen += 1
    assert seen >= 10, seen
