"""Builds libtbe.so (HIP, gfx950 only) in-tree with hipcc.

Every source is compiled on its own (in parallel) with the compiler's kernel-resource-usage
remarks switched on; the remarks are collected into `_build/resource_usage.txt` and checked
for the properties the library relies on:
  - `transfer_kernel` allocates at least 128 vector registers per lane (with 1024 threads per
    workgroup that fills a CU's register files, which is how the kernel keeps its CUs to itself);
  - no kernel spills registers to scratch memory.
The packed-fp32 target feature is switched off for the device pass.  hipcc hands `-Xclang` options
to the host pass as well, which does not know the feature and says so once per file and pass;
that one line is dropped from the output (everything else the compiler prints is shown).
"""
from __future__ import annotations

import concurrent.futures
import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libtbe.so")
SOURCES = ["tbe_api.hip", "tbe_sort.hip", "tbe_cache.hip", "tbe_move.hip", "tbe_embed.hip", "tbe_place.hip"]
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wno-unused-function"]
REMARKS = ["-Rpass-analysis=kernel-resource-usage"]
HARMLESS = "'-packed-fp32-ops' is not a recognized feature for this target (ignoring feature)"
MIN_VGPRS = {"transfer_kernel": 128}  # kernel-name substring -> fewest vector registers it must allocate

_REMARK = re.compile(r"remark:\s+(Function Name|TotalSGPRs|VGPRs|AGPRs|ScratchSize \[bytes/lane\]|Occupancy \[waves/SIMD\]|"
                     r"VGPRs Spill|SGPRs Spill|LDS Size \[bytes/block\]):\s+(\S+)")


def _demangle(names):
    try:
        out = subprocess.run(["c++filt"], input="\n".join(names), capture_output=True, text=True, check=True)
        res = out.stdout.split("\n")[:len(names)]
        return res if len(res) == len(names) else names
    except (OSError, subprocess.CalledProcessError):
        return names


def parse_resource_usage(stderr: str):
    """{mangled kernel name: {field: int}} from the compiler's remarks"""
    usage, cur = {}, None
    for line in stderr.splitlines():
        m = _REMARK.search(line)
        if not m:
            continue
        if m.group(1) == "Function Name":
            cur = usage.setdefault(m.group(2), {})
        elif cur is not None:
            try:
                cur[m.group(1)] = int(m.group(2))
            except ValueError:
                pass
    return usage


def _compile(hipcc: str, src: str, verbose: bool):
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    cmd = [hipcc] + FLAGS + REMARKS + ["-c", os.path.join(CSRC, src), "-o", obj]
    if verbose:
        print(" ".join(cmd), flush=True)
    p = subprocess.run(cmd, capture_output=True, text=True)
    return src, obj, p.returncode, p.stderr


def _is_remark_line(line: str, state: dict) -> bool:
    """remarks come as a line with `remark:` followed by two lines of source context"""
    if "[-Rpass-analysis=kernel-resource-usage]" in line:
        state["skip"] = 2
        return True
    if state.get("skip", 0) > 0:
        state["skip"] -= 1
        return True
    return False


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(6, os.cpu_count() or 1)) as ex:
        results = list(ex.map(lambda s: _compile(hipcc, s, verbose), SOURCES))
    usage, failed = {}, False
    for src, obj, rc, err in results:
        state = {}
        for line in err.splitlines():
            if line.strip() == HARMLESS or _is_remark_line(line, state):
                continue
            print(line, file=sys.stderr)
        failed |= rc != 0
        usage.update(parse_resource_usage(err))
    if failed:
        raise subprocess.CalledProcessError(1, "hipcc -c")
    names = list(usage)
    plain = dict(zip(names, _demangle(names)))
    with open(os.path.join(OBJ, "resource_usage.txt"), "w") as f:
        for n in sorted(names, key=lambda x: plain[x]):
            u = usage[n]
            f.write(f"{plain[n]}\n    VGPRs {u.get('VGPRs')} AGPRs {u.get('AGPRs')} SGPRs {u.get('TotalSGPRs')} "
                    f"occupancy {u.get('Occupancy [waves/SIMD]')} LDS {u.get('LDS Size [bytes/block]')} "
                    f"scratch {u.get('ScratchSize [bytes/lane]')} spills {u.get('VGPRs Spill')}/{u.get('SGPRs Spill')}\n")
    for n in names:
        u = usage[n]
        if u.get("VGPRs Spill", 0) or u.get("ScratchSize [bytes/lane]", 0):
            raise RuntimeError(f"build check: {plain[n]} spills to scratch memory ({u})")
        for sub, least in MIN_VGPRS.items():
            if sub in plain[n] and u.get("VGPRs", 0) < least:
                raise RuntimeError(f"build check: {plain[n]} allocates {u.get('VGPRs')} vector registers, needs {least}")
    for sub in MIN_VGPRS:
        if not any(sub in plain[n] for n in names):
            raise RuntimeError(f"build check: no resource remark for {sub}")
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + [obj for _, obj, _, _ in results] + ["-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
