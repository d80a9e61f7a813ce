"""Checks on the code hipcc generates for gfx950 (no GPU needed: the device code is compiled to assembly and read).

Why: one fault of this library was in no source line.  write_scalars, inlined at the end of a contraction kernel, once
had a return per version, each after its own stores; the compiler merged the versions' last store into one whose
address register one path never set (it held the flag output of a v_div_scale_f64), and that path stored to a stray
address.  The function now stores once per output; this test reads the generated code of every kernel that computes
the scalars - of every kernel, and every memory instruction whose address is an SGPR pair - and demands that no
definition by a flag, carry or mask output can reach such an address along the kernel's branches.
It also holds the kernels to their budgets: no private (scratch) memory, LDS within a compute unit's 160 KiB."""
from __future__ import annotations

import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2407_01445_amd", "csrc")
HIPCC = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
pytestmark = pytest.mark.skipif(not os.path.exists(HIPCC), reason="no hipcc")


NO_DEST = ("global_store", "flat_store", "buffer_store", "ds_write", "global_load_lds", "s_cmp", "s_cbranch", "s_branch",
           "s_waitcnt", "s_nop", "s_barrier", "s_endpgm", "s_bitcmp", "s_setprio", "s_sleep", "s_setpc", "s_sendmsg",
           "s_set", "s_icache", "s_dcache", "v_cmpx", "s_trap", "s_code_end")
SREG = re.compile(r"^s\[(\d+):(\d+)\]$|^s(\d+)$")


def sgprs_written(line: str):
    """SGPR ranges (lo, hi) an instruction writes: its first operand, and for vector instructions an SGPR pair in second
    place as well (the flag output of v_div_scale / the carry of v_add_co); vcc and exec are not tracked."""
    parts = line.strip().split(None, 1)
    if len(parts) < 2 or parts[0].startswith(NO_DEST) or parts[0].endswith(":"):
        return []
    ops = [o.strip() for o in parts[1].split(",")]
    out = []
    for pos, o in enumerate(ops[:2]):
        m = SREG.match(o)
        if not m or (pos == 1 and not parts[0].startswith("v_")):
            continue
        out.append((int(m.group(1)), int(m.group(2))) if m.group(1) else (int(m.group(3)), int(m.group(3))))
    return out


MASK_OPS = ("s_cselect_b64", "s_and_b64", "s_or_b64", "s_andn2_b64", "s_xor_b64", "s_orn2_b64", "s_and_saveexec_b64",
            "s_or_saveexec_b64")


def memory_instructions_with_stray_base(asm: str):
    """Every global_* / s_load_* instruction of every kernel of `asm` whose address is an SGPR pair: every definition of
    that pair that can REACH the instruction along the kernel's branches, followed through plain copies (s_mov_b64).  An
    address must come from the kernel arguments (s_load) or from scalar arithmetic on them; a definition by a vector
    instruction other than a lane read (a flag or carry output) or by a mask operation is a stray address.
    Returns (number of instructions checked, [(kernel, instruction, definition)] of stray ones)."""
    bad, checked = [], 0
    for m in re.finditer(r"^(_ZN2fc\w+):.*?(?=^\s*\.section)", asm, re.S | re.M):
        name, body = m.group(1), m.group(0)
        lines = [ln for ln in body.split("\n") if ln.strip() and not ln.lstrip().startswith(";")]
        label_at = {ln.strip()[:-1]: i for i, ln in enumerate(lines) if ln.strip().endswith(":")}
        preds = {i: [] for i in range(len(lines))}
        for i, ln in enumerate(lines):
            op = ln.strip().split(None, 1)
            falls = not (op[0] in ("s_branch", "s_endpgm") or op[0].startswith("s_setpc"))
            if op[0].startswith(("s_cbranch", "s_branch")) and len(op) > 1 and op[1].strip() in label_at:
                preds[label_at[op[1].strip()]].append(i)
            if falls and i + 1 < len(lines):
                preds[i + 1].append(i)

        def reaching(i, lo, hi, depth=0):
            """definitions of s[lo:hi] that reach the point BEFORE instruction i"""
            found, seen, work = [], set(), list(preds[i])
            while work:
                j = work.pop()
                if j in seen:
                    continue
                seen.add(j)
                if any(not (whi < lo or wlo > hi) for wlo, whi in sgprs_written(lines[j])):
                    ins = lines[j].strip()
                    cp = re.match(r"s_mov_b64\s+s\[\d+:\d+\],\s*s\[(\d+):(\d+)\]$", ins)
                    if cp and depth < 4:
                        found += reaching(j, int(cp.group(1)), int(cp.group(2)), depth + 1)
                    else:
                        found.append(ins)
                    continue
                work += preds[j]
            return found

        for i, ln in enumerate(lines):
            ins = ln.strip().split(None, 1)
            if len(ins) < 2 or not ins[0].startswith(("global_", "s_load_")):
                continue
            ops = [o.strip().split()[0] for o in ins[1].split(",") if o.strip()]
            cand = [ops[1]] if ins[0].startswith("s_load_") and len(ops) > 1 else ops[::-1]
            pair = next((SREG.match(o) for o in cand if SREG.match(o) and SREG.match(o).group(1)), None)
            if pair is None:
                continue
            checked += 1
            for d in reaching(i, int(pair.group(1)), int(pair.group(2))):
                op = d.split()[0]
                if (op.startswith("v_") and not op.startswith(("v_readlane", "v_readfirstlane"))) or op in MASK_OPS:
                    bad.append((name, ln.strip(), d))
    return checked, bad


def test_the_checker_sees_the_store_that_faulted():
    """The generated code that faulted, kept as a fixture: the merged last store can be reached with its address pair
    last written by a v_div_scale_f64 (the V3 path), besides the two good definitions (the loss and the d_tau pointer)."""
    asm = open(os.path.join(ROOT, "tests", "golden", "faulty_scalar_tail_gfx950.s")).read()
    checked, bad = memory_instructions_with_stray_base(asm)
    assert checked >= 4
    assert bad and all(b[1] == "global_store_dword v1, v0, s[4:5]" and b[2].startswith("v_div_scale_f64") for b in bad)


@pytest.fixture(scope="module")
def assembly(tmp_path_factory):
    out = {}
    d = tmp_path_factory.mktemp("isa")
    for src in sorted(f for f in os.listdir(CSRC) if f.endswith(".hip")):
        dst = str(d / (src[:-4] + ".s"))
        r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
                            "-packed-fp32-ops", "-I", os.path.join(ROOT, "include"), "-I", CSRC, "--cuda-device-only",
                            "-S", "-o", dst, os.path.join(CSRC, src)], capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-3000:]
        out[src] = open(dst).read()
    return out


def test_every_scalar_address_comes_from_the_kernel_arguments(assembly):
    """All kernels, every memory instruction whose address is an SGPR pair (1600 of them): none can be reached with
    that pair last written by a flag, carry or mask output."""
    total = 0
    for src, asm in assembly.items():
        checked, bad = memory_instructions_with_stray_base(asm)
        assert not bad, "%s: %s" % (src, bad[:5])
        total += checked
    assert total >= 1000


def test_no_kernel_uses_scratch_memory_and_lds_fits_a_compute_unit(assembly):
    n = 0
    for src, asm in assembly.items():
        for m in re.finditer(r"\.group_segment_fixed_size:\s*(\d+).*?\.name:\s*(\S+).*?\.private_segment_fixed_size:\s*(\d+)"
                             r".*?\.vgpr_spill_count:\s*(\d+)", asm, re.S):
            lds, name, scratch, spills = int(m.group(1)), m.group(2), int(m.group(3)), int(m.group(4))
            n += 1
            if "write_scalars" in name and "k_" not in name:
                continue                                     # a device function, not a kernel
            assert lds <= 160 * 1024, (name, lds)
            assert scratch == 0 and spills == 0, (name, scratch, spills)
    assert n >= 30
