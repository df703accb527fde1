"""Build libdecoquant.so in-tree with hipcc for gfx950."""
from __future__ import annotations

import glob
import json
import os
import re
import subprocess

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
LIB_PATH = os.path.join(PKG_DIR, "libdecoquant.so")
# registers, scratch and LDS of every kernel of the last build, as the compiler reported them
RESOURCES_PATH = os.path.join(PKG_DIR, "_build", "kernel_resources.json")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed-fp32 instructions are switched off for all device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # one remark per kernel with its register, scratch and LDS use (collected into RESOURCES_PATH)
    "-Rpass-analysis=kernel-resource-usage",
]


def sources():
    return sorted(glob.glob(os.path.join(PKG_DIR, "csrc", "*.hip")))


def _run(cmd):
    proc = subprocess.run(cmd, capture_output=True, text=True)
    log = "\n".join(l for l in (proc.stdout + proc.stderr).splitlines() if "packed-fp32-ops" not in l)
    return proc.returncode, log


_REMARK = re.compile(r"remark:\s+(Function Name|VGPRs|AGPRs|ScratchSize \[bytes/lane\]|VGPRs Spill|SGPRs Spill|"
                     r"LDS Size \[bytes/block\]|Occupancy \[waves/SIMD\]):\s*(\S+)")


def _split_remarks(log: str):
    """Separate the per-kernel resource remarks from the rest of a compiler log."""
    kernels, rest, name, after_remark = {}, [], None, False
    for line in log.splitlines():
        m = _REMARK.search(line)
        if after_remark and re.match(r"^\s*(\d+\s*)?\|", line):
            continue   # the source line and caret the compiler prints under a remark
        after_remark = bool(m) or "kernel-resource-usage" in line
        if m:
            key, val = m.group(1), m.group(2)
            if key == "Function Name":
                name = val
                kernels[name] = {}
            elif name is not None:
                kernels[name][key.split(" [")[0]] = int(val)
        elif "kernel-resource-usage" not in line:
            rest.append(line)
    if not any(("warning" in l) or ("error" in l) for l in rest):
        rest = []   # only the include trail that led to the remarks is left
    return kernels, "\n".join(rest)


TIMELINE_LIB_PATH = os.path.join(PKG_DIR, "libdecoquant_timeline.so")


def build_library(verbose: bool = False, timeline: bool = False) -> str:
    """Compile every HIP source (in parallel, one hipcc per file) and link one shared library;
    returns its path.  timeline=True builds the instrumented copy (-DDQ_TIMELINE: the matrix-core
    decode kernel stamps a time line per wave; see timeline.py) beside the product library, which it
    leaves alone."""
    from concurrent.futures import ThreadPoolExecutor
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    obj_dir = os.path.join(PKG_DIR, "_build_timeline" if timeline else "_build")
    os.makedirs(obj_dir, exist_ok=True)
    flags = [f for f in HIPCC_FLAGS if f != "-shared"] + (["-DDQ_TIMELINE"] if timeline else [])
    out_path = TIMELINE_LIB_PATH if timeline else LIB_PATH
    includes = ["-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(PKG_DIR, "csrc")]
    jobs = []
    for src in sources():
        obj = os.path.join(obj_dir, os.path.basename(src) + ".o")
        jobs.append((src, obj, [hipcc, *flags, *includes, "-c", src, "-o", obj]))
    workers = max(1, min(len(jobs), int(os.environ.get("MAX_JOBS", "8")), os.cpu_count() or 1))
    with ThreadPoolExecutor(workers) as pool:
        results = list(pool.map(lambda j: _run(j[2]), jobs))
    logs, resources = [], {}
    for (src, _, _), (rc, log) in zip(jobs, results):
        kernels, log = _split_remarks(log)
        if rc != 0:
            raise RuntimeError("hipcc failed on %s:\n%s" % (os.path.basename(src), log))
        resources.update(kernels)
        logs.append(log)
    if not timeline:
        with open(RESOURCES_PATH, "w") as f:
            json.dump(resources, f, indent=0, sort_keys=True)
    rc, log = _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *[j[1] for j in jobs], "-o", out_path + ".tmp"])
    if rc != 0:
        raise RuntimeError("link failed:\n" + log)
    os.replace(out_path + ".tmp", out_path)
    if verbose and any(l.strip() for l in logs + [log]):
        print("\n".join(l for l in logs + [log] if l.strip()))
    return out_path


if __name__ == "__main__":
    import sys
    print(build_library(verbose=True, timeline="--timeline" in sys.argv))
