"""Builds the CPU emulation of libfastclip: the library's own sources compiled for the host against the stand-in
hip/hip_runtime.h of this folder, linked with emu_main.cpp into _build/emu/emu_step, AddressSanitizer on.

The sources are copied with the few constructs a host compiler cannot take replaced by calls into the stand-in: inline
assembly (direct-to-LDS loads, accumulator reads) and the LDS address-space attribute.  Nothing else differs: indexing,
guards, barriers and the order of operations are the product's."""
from __future__ import annotations

import os
import re
import shutil
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
CSRC = os.path.join(ROOT, "paper_2407_01445_amd", "csrc")
OUT = os.path.join(ROOT, "_build", "emu")
EXE = os.path.join(OUT, "emu_step")


def host_compiler():
    for c in ("/opt/rocm/llvm/bin/clang++", shutil.which("clang++")):
        if c and os.path.exists(c):
            return c
    return None


def _asm_replacement(m):
    t = m.group(0)
    if "s_add_u32 m0" in t:                      # 16 bytes per lane into LDS at (uniform + IMM) + 16 lane
        return "emu_dma(uniform_base, lane_byte_off, lds_uniform + (uint32_t)IMM, 16);"
    if "global_load_lds_dwordx4" in t:
        return "emu_dma(uniform_base, lane_byte_off, lds_byte_addr, 16);"
    if "global_load_lds_dword " in t:
        return "emu_dma(uniform_base, lane_byte_off, lds_byte_addr, 4);"
    if "v_accvgpr_read_b32" in t:
        return "x = in_agpr;"
    if re.search(r'asm volatile\(""', t):         # keeps a value alive, nothing to run
        return "(void)0;"
    raise RuntimeError("inline assembly the emulation does not know: " + t)


def generate():
    gen = os.path.join(OUT, "gen")
    os.makedirs(gen, exist_ok=True)
    units = []
    for d, names in ((CSRC, sorted(os.listdir(CSRC))), (os.path.join(ROOT, "include"), ["fastclip.h"])):
        for n in names:
            if not n.endswith((".hip", ".hpp", ".h")):
                continue
            s = open(os.path.join(d, n)).read()
            s = s.replace("__attribute__((address_space(3)))", "")
            s = re.sub(r'asm volatile\((?:[^;]|\n)*?\);', _asm_replacement, s)
            out = os.path.join(gen, n.replace(".hip", ".inc"))
            open(out, "w").write(s)
            if n.endswith(".hip"):
                units.append(out)
    return gen, units


def build(sanitizer: str = "-fsanitize=address") -> str:
    cxx = host_compiler()
    if cxx is None:
        raise RuntimeError("no host clang++")
    gen, units = generate()
    obj = os.path.join(OUT, "obj")
    os.makedirs(obj, exist_ok=True)
    flags = ["-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", sanitizer, "-I", HERE, "-I", gen, "-pthread",
             "-Wno-unused-value", "-Wno-ignored-attributes"]

    def one(src):
        o = os.path.join(obj, os.path.basename(src).rsplit(".", 1)[0] + ".o")
        r = subprocess.run([cxx, *flags, "-x", "c++", "-c", src, "-o", o], capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("host build of %s failed:\n%s" % (src, r.stderr[-4000:]))
        return o

    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(one, units + [os.path.join(HERE, "emu_main.cpp")]))
    r = subprocess.run([cxx, *flags, *objs, "-o", EXE], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr[-4000:])
    return EXE


if __name__ == "__main__":
    import sys
    print(build(*sys.argv[1:2]))
