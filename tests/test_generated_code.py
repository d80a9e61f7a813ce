"""Checks on the code hipcc generates for gfx950 (no GPU needed: the device code is compiled to assembly and read).

Why: one fault of this library was in no source line.  write_scalars, inlined at the end of a contraction kernel, once
had a return per version, each after its own stores; the compiler merged the versions' last store into one whose
address register one path never set (it held the flag output of a v_div_scale_f64), and that path stored to a stray
address.  The function now stores once per output; this test reads the generated code of every kernel that computes
the scalars and demands that each scalar store goes through a register pair loaded straight from the kernel arguments.
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


def scalar_stores_with_stray_address(asm: str):
    """For every kernel of `asm` that divides in fp64 and stores single dwords through an SGPR address pair after its
    first fp64 reciprocal (the tail that computes the step's scalars): every definition of that pair that can REACH the
    store along the kernel's branches, followed through plain copies (s_mov_b64).  An address must come from the kernel
    arguments (s_load) or from scalar arithmetic on them; a definition by a vector instruction (a flag or mask output)
    or by a mask operation is a stray address.  Returns (kernel, store, definition) triples of stray ones."""
    bad = []
    for m in re.finditer(r"^(_ZN2fc\w+):.*?(?=^\s*\.section)", asm, re.S | re.M):
        name, body = m.group(1), m.group(0)
        if "v_div_fixup_f64" not in body:
            continue
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

        first = next(i for i, ln in enumerate(lines) if "v_rcp_f64" in ln)
        for i in range(first, len(lines)):
            st = re.match(r"\s*global_store_dword\s+\S+,\s*\S+,\s*s\[(\d+):(\d+)\]", lines[i])
            if not st:
                continue
            for d in reaching(i, int(st.group(1)), int(st.group(2))):
                op = d.split()[0]
                stray = op.startswith("v_") or op in ("s_cselect_b64", "s_and_b64", "s_or_b64", "s_andn2_b64", "s_xor_b64",
                                                      "s_orn2_b64", "s_and_saveexec_b64", "s_or_saveexec_b64")
                if stray:
                    bad.append((name, lines[i].strip(), d))
    return bad


def test_the_checker_sees_the_store_that_faulted():
    """The generated code that faulted, kept as a fixture: the merged last store can be reached with its address pair
    last written by a v_div_scale_f64 (the V3 path), besides the two good definitions (the loss and the d_tau pointer)."""
    asm = open(os.path.join(ROOT, "tests", "golden", "faulty_scalar_tail_gfx950.s")).read()
    bad = scalar_stores_with_stray_address(asm)
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


def test_scalar_stores_go_through_the_pointers_the_kernel_was_given(assembly):
    seen = 0
    for src, asm in assembly.items():
        bad = scalar_stores_with_stray_address(asm)
        assert not bad, "%s: %s" % (src, bad)
        seen += sum(1 for m in re.finditer(r"^(_ZN2fc\w+):.*?(?=^\s*\.section)", asm, re.S | re.M)
                    if "v_div_fixup_f64" in m.group(0))
    assert seen >= 6        # the finishing kernels of every path and the scalars' own kernel


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
