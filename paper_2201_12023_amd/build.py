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
        for key, pat in (("vgprs", r" VGPRs: (\d+)"), ("scratch", r"ScratchSize \[bytes/lane\]: (\d+)"),
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

    with ThreadPoolExecutor(max_workers=4) as ex:
        list(ex.map(cc, zip(srcs, objs)))
    bad = check_resources(kernels)
    if bad:
        raise RuntimeError("register budget of the recurrence kernel not met:\n  " + "\n  ".join(bad))
    if verbose:
        n_batch = sum(1 for k in kernels if _BATCH_INSTANCE.search(k))
        print(f"resource check: {len(kernels)} kernels, {n_batch} batch instances at 8 waves/SIMD, "
              "no scratch in the recurrence kernel", flush=True)
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    build(extra=sys.argv[1:])
