"""Build step for the HIP library: hipcc, gfx950 only, in-tree output.

``python -m paper_2201_12023_amd.build`` compiles every ``csrc/*.hip`` into
``paper_2201_12023_amd/libalpa_dp.so``.
"""
from __future__ import annotations

import glob
import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libalpa_dp.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]


# The batch form of the recurrence kernel (one candidate per workgroup, up to 64 layers) is
# built around eight waves per SIMD: 64 vector registers at most and nothing in scratch memory.
# The compiler only promises seven (see the kernel's attribute), so the register count of these
# instances is checked after every build instead of being found out on the GPU.
_BATCH_INSTANCE = re.compile(r"recurrence_fast_kernelILi[1-4]ELi1ELi1ELb0ELb0ELb0ELb0E")


def parse_resource_remarks(text: str) -> dict:
    """{mangled kernel name: {"vgprs", "scratch", "occupancy"}} from the compiler's
    -Rpass-analysis=kernel-resource-usage remarks."""
    out, cur = {}, None
    for line in text.splitlines():
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            cur = out.setdefault(m.group(1), {})
            continue
        if cur is None:
            continue
        for key, pat in (("vgprs", r" VGPRs: (\d+)"), ("agprs", r" AGPRs: (\d+)"),
                         ("scratch", r"ScratchSize \[bytes/lane\]: (\d+)"),
                         ("occupancy", r"Occupancy \[waves/SIMD\]: (\d+)")):
            m = re.search(pat, line)
            if m:
                cur[key] = int(m.group(1))
    return out


def check_resources(kernels: dict) -> list:
    """Violations of what the hot kernels are built around (empty list: fine)."""
    bad = []
    for name, r in sorted(kernels.items()):
        if _BATCH_INSTANCE.search(name):
            if r.get("occupancy", 0) < 8 or r.get("scratch", 0) != 0:
                bad.append(f"{name}: {r} (batch instance: 8 waves/SIMD and no scratch expected)")
        elif "recurrence_fast_kernel" in name and r.get("scratch", 0) != 0:
            bad.append(f"{name}: {r} (scratch memory in the recurrence kernel)")
        # The kernel's warm-up loads land in a vector register that must stay where it is while
        # they are in flight (it is tied through inline asm from the loads to a wait at the end
        # of the ticket).  What could move it is a spill, to scratch memory or to an
        # accumulation register: neither may appear.
        if "recurrence_fast_kernel" in name and r.get("agprs", 0) != 0:
            bad.append(f"{name}: {r} (accumulation registers in the recurrence kernel: a spill)")
    return bad


def check_warm_register(asm_text: str) -> list:
    """The same guard at the level of the emitted code.  For every recurrence_fast_kernel in
    the device assembly: the inline-asm warm-up loads all land in one vector register, a
    closing `s_waitcnt vmcnt(0)` follows them, and between the first of the loads and that wait
    (text order: the layer bodies lie in between) nothing but the loads themselves and
    `v_mov_b32 <it>, 0` writes that register."""
    bad = []
    for part in re.split(r"\n(?=_ZN4alpa22recurrence_fast_kernel\S*:)", asm_text)[1:]:
        name = part.split(":", 1)[0]
        lines = part[:part.find("s_endpgm")].splitlines()
        in_asm, loads, waits, asm_lines = False, [], [], set()
        for i, line in enumerate(lines):
            t = line.strip()
            if t.startswith(";;#ASMSTART"):
                in_asm = True
            elif t.startswith(";;#ASMEND"):
                in_asm = False
            elif in_asm:
                asm_lines.add(i)
                m = re.match(r"global_load_dword (v\d+),", t)
                if m:
                    loads.append((i, m.group(1)))
                if "s_waitcnt vmcnt(0)" in t:
                    waits.append(i)
        if not loads:
            continue
        regs = sorted({r for _, r in loads})
        if len(regs) != 1:
            bad.append(f"{name}: warm-up loads land in {regs}")
            continue
        reg, num = regs[0], int(regs[0][1:])
        first = loads[0][0]
        closing = [w for w in waits if w > loads[-1][0]]
        if not closing:
            bad.append(f"{name}: no wait behind the warm-up loads")
            continue
        for i in range(first, closing[0]):
            if i in asm_lines:
                continue
            t = lines[i].strip()
            m = re.match(r"(v_\w+|ds_read\w*|global_load\w*|buffer_load\w*|scratch_load\w*)\s+([^,\s]+)", t)
            if not m or m.group(1).startswith(("v_cmp", "v_readlane", "v_readfirstlane")):
                continue
            dst = m.group(2)
            span = re.match(r"v\[(\d+):(\d+)\]", dst)
            hit = dst == reg or (span and int(span.group(1)) <= num <= int(span.group(2)))
            if hit and not re.match(rf"v_mov_b32_e32 {reg}, 0$", t):
                bad.append(f"{name}: `{t}` writes {reg} while warm-up loads may be in flight")
    return bad


def build(verbose: bool = True, extra=()) -> str:
    os.makedirs(OBJ, exist_ok=True)
    srcs = sorted(glob.glob(os.path.join(CSRC, "*.hip")))
    objs = [os.path.join(OBJ, os.path.basename(s)[:-4] + ".o") for s in srcs]
    kernels = {}

    def cc(pair):
        s, o = pair
        cmd = [HIPCC, *FLAGS, *extra, "-Rpass-analysis=kernel-resource-usage", "-c", s, "-o", o]
        if verbose:
            print(" ".join(cmd), flush=True)
        res = subprocess.run(cmd, stderr=subprocess.PIPE, text=True)
        rest = [l for l in res.stderr.splitlines() if "-Rpass-analysis=kernel-resource-usage" not in l]
        if rest and (verbose or res.returncode):
            print("\n".join(rest), file=sys.stderr, flush=True)
        if res.returncode:
            raise subprocess.CalledProcessError(res.returncode, cmd)
        kernels.update(parse_resource_remarks(res.stderr))

    # device assembly of the two files that instantiate the recurrence kernel, for the check above
    asm_jobs = [(s, os.path.join(OBJ, os.path.basename(s)[:-4] + ".s")) for s in srcs
                if os.path.basename(s).startswith("kernels_fast")]
    asm_bad = []

    def asm(pair):
        s, o = pair
        cmd = [HIPCC, *[f for f in FLAGS if f not in ("-fPIC",)], *extra, "--cuda-device-only", "-S", s, "-o", o]
        if verbose:
            print(" ".join(cmd), flush=True)
        res = subprocess.run(cmd, stderr=subprocess.PIPE, text=True)
        if res.returncode:
            print(res.stderr, file=sys.stderr, flush=True)
            raise subprocess.CalledProcessError(res.returncode, cmd)
        with open(o) as f:
            asm_bad.extend(check_warm_register(f.read()))
        os.remove(o)

    with ThreadPoolExecutor(max_workers=4) as ex:
        jobs = [ex.submit(cc, p) for p in zip(srcs, objs)] + [ex.submit(asm, p) for p in asm_jobs]
        for j in jobs:
            j.result()
    bad = check_resources(kernels) + asm_bad
    if bad:
        raise RuntimeError("register budget of the recurrence kernel not met:\n  " + "\n  ".join(bad))
    if verbose:
        n_batch = sum(1 for k in kernels if _BATCH_INSTANCE.search(k))
        print(f"resource check: {len(kernels)} kernels, {n_batch} batch instances at 8 waves/SIMD, "
              "no spills in the recurrence kernel, its warm-up register keeps its place", flush=True)
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    build(extra=sys.argv[1:])
