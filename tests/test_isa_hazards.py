"""Static check of the generated gfx950 code of the GEMV kernels (no GPU needed).

The inner blocks are inline assembly that ends in v_dot2c_f32_f16 instructions.  On this
architecture a dot-product result may feed the next dot product at once, but any other
instruction that reads it needs three wait states in between, and the compiler's hazard
pass cannot see instructions inside an asm statement.  The kernels therefore put a
s_nop after every consume step; this test compiles the kernels to assembly and verifies
that no compiler-generated instruction (e.g. a register copy of an accumulator at a
loop boundary) reads a dot2c destination too early.
"""
import os
import re
import shutil
import subprocess

import pytest

from paper_2402_15319_amd import build as vqbuild

WAIT_STATES = 3


def _regs(tok):
    out = set()
    for m in re.finditer(r"v\[(\d+):(\d+)\]|\bv(\d+)\b", tok):
        if m.group(3) is not None:
            out.add(int(m.group(3)))
        else:
            out.update(range(int(m.group(1)), int(m.group(2)) + 1))
    return out


def scan(lines):
    """Returns [(line number, text)] of instructions that read a dot2c result too early."""
    bad = []
    recent = []   # (registers written by a dot2c, wait states since)
    for ln, line in enumerate(lines, 1):
        t = line.split(";")[0].strip()
        if not t or t.startswith(".") or t.endswith(":"):
            continue
        op, _, rest = t.partition(" ")
        ops = [o.strip() for o in rest.split(",")]
        if op == "s_nop":
            n = int(ops[0]) + 1
            recent = [(d, w + n) for d, w in recent if w + n < WAIT_STATES]
            continue
        if op.startswith("v_dot2c"):
            recent = [(d, w + 1) for d, w in recent if w + 1 < WAIT_STATES] + [(_regs(ops[0]), 0)]
            continue
        if op.startswith("v_"):
            src = set().union(*[_regs(o) for o in ops[1:]]) if len(ops) > 1 else set()
        elif op.startswith(("ds_", "global_", "buffer_", "flat_", "scratch_")):
            src = set().union(*[_regs(o) for o in ops])
        else:
            src = set()
        for d, w in recent:
            if d & src:
                bad.append((ln, t))
        recent = [(d, w + 1) for d, w in recent if w + 1 < WAIT_STATES]
    return bad


def test_scan_flags_an_early_read_and_accepts_a_fenced_one():
    early = ["v_dot2c_f32_f16 v3, v10, v11", "v_mov_b32_e32 v20, v3"]
    chained = ["v_dot2c_f32_f16 v3, v10, v11", "v_dot2c_f32_f16 v3, v12, v11"]
    fenced = ["v_dot2c_f32_f16 v3, v10, v11", "s_nop 3", "v_mov_b32_e32 v20, v3"]
    spaced = ["v_dot2c_f32_f16 v3, v10, v11", "v_add_u32_e32 v1, v2, v4", "s_mov_b32 s1, s2",
              "ds_read_b32 v5, v6", "v_mov_b32_e32 v20, v3"]
    other = ["v_dot2c_f32_f16 v3, v10, v11", "v_mov_b32_e32 v20, v31", "v_mov_b32_e32 v3, v30"]
    pair = ["v_dot2c_f32_f16 v3, v10, v11", "global_store_dwordx2 v[8:9], v[2:3], off"]
    assert len(scan(early)) == 1
    assert scan(chained) == []
    assert scan(fenced) == []
    assert scan(spaced) == []
    assert scan(other) == []
    assert len(scan(pair)) == 1


SWAP_WAIT_STATES = 2


def scan_swaps(lines):
    """Lane-swap instructions (v_permlane16_swap / v_permlane32_swap) sit in asm statements too: a
    vector instruction that writes one of their operands needs two wait states before the swap,
    and so does a vector instruction that reads a swapped register afterwards.  Returns
    [(line number, text)] of the swaps, or of the readers, that come too early."""
    bad = []
    writes = []   # (registers written by a vector instruction, wait states since)
    swaps = []    # (registers written by a swap, wait states since)
    for ln, line in enumerate(lines, 1):
        t = line.split(";")[0].strip()
        if not t or t.startswith(".") or t.endswith(":"):
            continue
        op, _, rest = t.partition(" ")
        ops = [o.strip() for o in rest.split(",")]
        if op == "s_nop":
            n = int(ops[0]) + 1
            writes = [(d, w + n) for d, w in writes if w + n < SWAP_WAIT_STATES]
            swaps = [(d, w + n) for d, w in swaps if w + n < SWAP_WAIT_STATES]
            continue
        is_swap = op.startswith(("v_permlane16_swap", "v_permlane32_swap"))
        regs_all = set().union(*[_regs(o) for o in ops]) if ops else set()
        if is_swap:
            if any(d & regs_all for d, _ in writes):
                bad.append((ln, t))
        elif op.startswith("v_") or op.startswith(("ds_", "global_", "buffer_", "flat_", "scratch_")):
            src = set().union(*[_regs(o) for o in ops[1:]]) if op.startswith("v_") and len(ops) > 1 else \
                (regs_all if not op.startswith("v_") else set())
            if any(d & src for d, _ in swaps):
                bad.append((ln, t))
        writes = [(d, w + 1) for d, w in writes if w + 1 < SWAP_WAIT_STATES]
        swaps = [(d, w + 1) for d, w in swaps if w + 1 < SWAP_WAIT_STATES]
        if is_swap:
            swaps.append((regs_all, 0))
        elif op.startswith("v_") and ops and not op.startswith("v_cmp"):
            writes.append((_regs(ops[0]), 0))
    return bad


def test_scan_swaps_flags_missing_wait_states():
    ok = ["v_add_f32_e32 v1, v2, v3", "s_nop 1", "v_permlane32_swap_b32_e32 v1, v4", "s_nop 1", "v_add_f32_e32 v5, v1, v4"]
    early_swap = ["v_add_f32_e32 v1, v2, v3", "s_nop 0", "v_permlane32_swap_b32_e32 v1, v4", "s_nop 1", "v_add_f32_e32 v5, v1, v4"]
    early_read = ["v_add_f32_e32 v1, v2, v3", "s_nop 1", "v_permlane16_swap_b32_e32 v1, v4", "s_nop 0", "v_add_f32_e32 v5, v9, v4"]
    unrelated = ["v_add_f32_e32 v7, v2, v3", "v_permlane16_swap_b32_e32 v1, v4", "v_add_f32_e32 v5, v9, v8"]
    assert scan_swaps(ok) == []
    assert len(scan_swaps(early_swap)) == 1
    assert len(scan_swaps(early_read)) == 1
    assert scan_swaps(unrelated) == []


@pytest.mark.skipif(shutil.which(os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")) is None,
                    reason="hipcc not available")
def test_no_instruction_reads_a_dot2c_result_early(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    out = tmp_path / "vq_gemv.s"
    flags = [f for f in vqbuild.HIPCC_FLAGS if f != "-fPIC"]
    cmd = [hipcc, *flags, "-S", "--cuda-device-only", "-o", str(out),
           os.path.join(vqbuild.CSRC, "vq_gemv.hip")]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-2000:]
    lines = out.read_text().splitlines()
    assert sum("v_dot2c_f32_f16" in l for l in lines) > 100     # the kernels are in there
    bad = scan(lines)
    assert bad == [], bad[:10]
    assert sum("v_permlane32_swap" in l for l in lines) > 10    # the reductions are in there
    bad = scan_swaps(lines)
    assert bad == [], bad[:10]


@pytest.mark.skipif(shutil.which(os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")) is None,
                    reason="hipcc not available")
def test_wide_group_kernels_read_no_dot2c_result_early(tmp_path):
    """The same two checks on the kernels of the formats whose tables are shared by 64 rows or more
    (d = 4: compiler-scheduled dot products; k = 256 with int8 tables: the hand-scheduled block)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    out = tmp_path / "vq_gemv_d4.s"
    flags = [f for f in vqbuild.HIPCC_FLAGS if f != "-fPIC"]
    cmd = [hipcc, *flags, "-S", "--cuda-device-only", "-o", str(out),
           os.path.join(vqbuild.CSRC, "vq_gemv_d4.hip")]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-2000:]
    lines = out.read_text().splitlines()
    assert sum("v_dot2c_f32_f16" in l for l in lines) >= 32 + 32   # both kernels' dot products are in there
    assert scan(lines) == []
    assert scan_swaps(lines) == []


@pytest.mark.skipif(shutil.which(os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")) is None,
                    reason="hipcc not available")
def test_e_step_kernel_has_no_fused_multiply_add(tmp_path):
    """The E-step's distance is defined with every operation rounded on its own (the CPU
    oracle takes the same decision with the same roundings); a contraction into a fused
    multiply-add would change near-ties.  Checks the generated code of the assign kernels."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    out = tmp_path / "vq_em.s"
    flags = [f for f in vqbuild.HIPCC_FLAGS if f != "-fPIC"]
    cmd = [hipcc, *flags, "-S", "--cuda-device-only", "-o", str(out), os.path.join(vqbuild.CSRC, "vq_em.hip")]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-2000:]
    inside, seen, fused = False, 0, []
    for line in out.read_text().splitlines():
        if re.match(r"^_ZN.*em_assign(_any)?_kernel.*:", line):
            inside, seen = True, seen + 1
        elif inside and "s_endpgm" in line:
            inside = False
        elif inside and re.match(r"\s+v_(fma|fmac|mac|mad|pk_fma|pk_mul|pk_add)_f32", line):
            fused.append(line.strip())
    assert seen == 3 + 25 + 10 + 6        # d = 2, 8-row groups: k = 16, 64, 256; 25 kernels for the other (k, d, group) cases; 10 for 4-row groups; 6 for k = 32
    assert fused == []
