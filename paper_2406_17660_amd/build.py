"""Build paper_2406_17660_amd/libgrass.so from csrc/*.hip with hipcc for gfx950, and the
benchmark's measurement aid probe/libgrass_probe.so from probe/*.hip.

The libraries are built in-tree so that they travel with the source tree; tests, the smoke
check and the benchmark only load them.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libgrass.so")
PROBE_DIR = os.path.join(HERE, "probe")
PROBE_LIB = os.path.join(PROBE_DIR, "libgrass_probe.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# -packed-fp32-ops is switched off: the compiler must not form packed fp32 instructions.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function", "-Wno-inline-asm",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-ffp-contract=on"]


def sources(folder=CSRC):
    return sorted(os.path.join(folder, f) for f in os.listdir(folder) if f.endswith(".hip"))


def _compile(src: str) -> str:
    obj = os.path.join(OBJ_DIR, os.path.basename(src)[:-4] + ".o")
    cmd = [HIPCC, *FLAGS, "-c", src, "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in res.stderr.splitlines() if "is not a recognized feature" not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def _link(lib: str, objs) -> None:
    res = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs],
                         capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n" + res.stderr)


def build(verbose: bool = False) -> str:
    """Compile every .hip file (always: this is also the 'does it build' check) and link the
    two libraries."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    lib_src, probe_src = sources(CSRC), sources(PROBE_DIR)
    with ThreadPoolExecutor(max_workers=8) as pool:
        objs = list(pool.map(_compile, lib_src + probe_src))
    _link(LIB, objs[:len(lib_src)])
    _link(PROBE_LIB, objs[len(lib_src):])
    if verbose:
        print(LIB)
        print(PROBE_LIB)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
