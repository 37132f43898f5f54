"""Build tests/native/abi_smoke.bin: a C++ program that uses libgrass.so through its C ABI alone
(no Python, no torch) and checks itself against the oracle library.  Test infrastructure."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
OUT = os.path.join(HERE, "abi_smoke.bin")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def build() -> str:
    lib_dir = os.path.join(ROOT, "paper_2406_17660_amd")
    ref_dir = os.path.join(ROOT, "oracle")
    for need in (os.path.join(lib_dir, "libgrass.so"), os.path.join(ref_dir, "libgrass_ref.so")):
        if not os.path.exists(need):
            raise RuntimeError(f"{need} is missing: build the library and the oracle first")
    cmd = [HIPCC, "--offload-arch=gfx950", "-O2", "-std=c++17", os.path.join(HERE, "abi_smoke.cpp"),
           "-o", OUT, f"-L{lib_dir}", f"-L{ref_dir}", "-lgrass", "-lgrass_ref",
           "-Wl,-rpath,$ORIGIN/../../paper_2406_17660_amd:$ORIGIN/../../oracle"]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("building abi_smoke failed:\n" + res.stderr)
    return OUT


if __name__ == "__main__":
    print(build())
