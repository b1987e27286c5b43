"""Build libkvc.so for gfx950 with hipcc (cross-compiles without a GPU).

After compiling, the device assembly of every kernel is checked for one instruction form that this
GPU executes wrongly and this compiler does not avoid for gfx950: a 64-bit shift (v_lshlrev_b64,
v_lshrrev_b64, v_ashrrev_i64) whose shift count is the last VGPR of the wave's allocation (register
number 8n+7 with no allocated register after it).  Four waves per SIMD of a kernel with
`v_lshlrev_b64 v[a:b], v111, v[c:d]` and 112 registers shifted by the lane number instead of the
count in about one execution of eight (a stand-alone kernel that does nothing else shows it; with
120 registers allocated, or the count in v109, it never does).  LLVM describes and works around
the same fault for gfx90a only.  A kernel that trips the check gets register headroom: an empty
asm statement naming a higher register (see decode_kernel).
"""
import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
OUT = os.path.join(HERE, "libkvc.so")
WIDTHS = (2, 3, 4, 8)
# (source, code width or None): the kernel sources are compiled once per code width, which spreads
# the build over the cores; the slowest units come first
JOBS = ([("kvc_huff_enc.hip", b) for b in WIDTHS] + [("kvc_quant.hip", b) for b in WIDTHS] +
        [("kvc_huff_dec.hip", b) for b in WIDTHS] +
        [("kvc_huff_tables.hip", None), ("kvc_selftest.hip", None), ("kvc_service.hip", None), ("kvc_probe.hip", None),
         ("kvc_api.hip", None), ("kvc_policy.hip", None)])
# packed fp32 instructions are switched off for the device pass (flag for hipcc only)
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall",
         "-Wno-unused-command-line-argument"]


def shift_count_in_last_vgpr(asm_path):
    """[(kernel symbol, instruction)] for 64-bit shifts that take their count from the last
    allocated VGPR, read from the device assembly hipcc leaves with -save-temps."""
    text = open(asm_path).read()
    next_free = {k: int(re.search(r"\.amdhsa_next_free_vgpr (\d+)", body).group(1))
                 for k, body in re.findall(r"\.amdhsa_kernel (\w+)\n(.*?)\.end_amdhsa_kernel", text, re.S)}
    shift = re.compile(r"\s+v_(?:lshlrev_b64|lshrrev_b64|ashrrev_i64)\s+v\[\d+:\d+\],\s*v(\d+),")
    hits, cur = [], None
    for line in text.split("\n"):
        m = re.match(r"^(\w+):", line)
        if m and m.group(1) in next_free:
            cur = m.group(1)                         # a kernel's code starts at its symbol ...
        elif line.startswith(".Lfunc_end"):
            cur = None                               # ... and ends here
        elif cur is not None:
            m = shift.match(line)
            if m and int(m.group(1)) % 8 == 7 and int(m.group(1)) + 1 >= next_free[cur]:
                hits.append((cur, line.strip()))
    return hits


def spilling_kernels(asm_path):
    """[(kernel symbol, scratch bytes per lane)] of the kernels that spill registers."""
    text = open(asm_path).read()
    out = []
    for k, body in re.findall(r"\.amdhsa_kernel (\w+)\n(.*?)\.end_amdhsa_kernel", text, re.S):
        n = int(re.search(r"\.amdhsa_private_segment_fixed_size (\d+)", body).group(1))
        if n:
            out.append((k, n))
    return out


def _compile(job):
    name, width = job
    stem = name.replace(".hip", "") + ("_b%d" % width if width else "")
    # -save-temps names its files after the source, so every job works on a copy named after itself
    src = os.path.join(OBJ, stem + ".hip")
    with open(src, "w") as f:
        f.write('#include "%s"\n' % os.path.join(SRC, name))
    obj = os.path.join(OBJ, stem + ".o")
    cmd = ["hipcc"] + FLAGS + (["-DKVC_BITS=%d" % width] if width else []) + ["-I", SRC, "-save-temps=obj", "-c", src, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (name, err))
    name = stem
    asm = os.path.join(OBJ, stem + "-hip-amdgcn-amd-amdhsa-gfx950.s")
    hits = shift_count_in_last_vgpr(asm)
    if hits:
        raise RuntimeError("%s: 64-bit shift with its count in the last allocated VGPR (give the kernel register "
                           "headroom):\n%s" % (name, "\n".join("  %s: %s" % h for h in hits[:20])))
    spills = spilling_kernels(asm)
    if spills:
        err += "\n%s: %d kernels spill registers (most: %d bytes per lane): %s" % (
            name, len(spills), max(n for _, n in spills), ", ".join(k for k, _ in spills[:6]))
    for f in os.listdir(OBJ):                      # the temporaries are large and no longer needed
        if (f.startswith(stem + "-") or f.startswith(stem + ".hip-")) and f != stem + ".o":
            os.remove(os.path.join(OBJ, f))
    return obj, err


def build(verbose=False):
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 4)) as ex:
        results = list(ex.map(_compile, JOBS))
    if verbose:
        for _, err in results:
            if err.strip():
                print(err)
    objs = [o for o, _ in results]
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", OUT] + objs)
    return OUT


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
