"""Builds (hipcc, gfx950) and runs the microbenchmarks whose results shaped the kernels:
`python -m paper_2502_02406_amd.microbench [--build-only]`.  Their sources say what each measures;
the numbers of one run are kept in profiles/hardware_microbenchmarks.md."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
BIN = os.path.join(HERE, "bin")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]
PROGRAMS = ["dq_exchange", "vm_order"]


def build() -> None:
    os.makedirs(BIN, exist_ok=True)
    for name in PROGRAMS:
        src, exe = os.path.join(HERE, name + ".hip"), os.path.join(BIN, name)
        if os.path.exists(exe) and os.path.getmtime(exe) >= os.path.getmtime(src):
            continue
        r = subprocess.run([HIPCC] + FLAGS + [src, "-o", exe], capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed for {src}:\n{r.stdout}{r.stderr}")


if __name__ == "__main__":
    build()
    if "--build-only" not in sys.argv:
        for name in PROGRAMS:
            print(f"==== {name}", flush=True)
            subprocess.run([os.path.join(BIN, name)], check=True, timeout=300)
