"""Build liblvx.so (the C-ABI HIP library) for gfx950, in-tree, with hipcc.

    python -m paper_2502_02406_amd.build

Every translation unit under csrc/ is compiled with
``hipcc --offload-arch=gfx950 -O3`` and linked into ``paper_2502_02406_amd/liblvx.so``.
hipcc cross-compiles, so this runs on machines without a GPU.
"""
from __future__ import annotations

import glob
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "liblvx.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         # hipcc may fuse scalar float math into packed-fp32 instructions; keep them off
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument",
         # the tile-copy statements name m0 as clobbered on purpose (they load it with the LDS
         # address); clang notes for every use that it does not preserve a reserved register
         "-Wno-inline-asm"]


# Per-file flags.  The key-stationary backward kernel runs one wave per SIMD with the whole
# register file; there the compiler would by default put every matrix-instruction result into the
# accumulation registers, including the scores that the vector ALU consumes next.  Its own
# accumulators are pinned to that file in the source, everything else stays in ordinary registers.
FILE_FLAGS = {"lvx_bwd_dkdv_bf16.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"],
              # (its contraction phase is one unrolled run of 48 matrix instructions with the vector work
              # of a step between them: larger than what the unroll pragma accepts by default)
              "lvx_bwd_fused_bf16.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1",
                                         "-mllvm", "-pragma-unroll-threshold=200000"]}


def _compile(src: str, force: bool, extra) -> str:
    obj = os.path.join(OBJ, os.path.basename(src).replace(".hip", ".o"))
    deps = [src] + glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(HERE, "..", "include", "*.h"))
    if not force and os.path.exists(obj) and all(os.path.getmtime(obj) >= os.path.getmtime(d) for d in deps):
        return obj
    cmd = [HIPCC] + FLAGS + FILE_FLAGS.get(os.path.basename(src), []) + list(extra) + ["-c", src, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    msgs = "\n".join(l for l in (r.stdout + r.stderr).splitlines()
                     if "packed-fp32-ops" not in l and l.strip())
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{msgs}")
    if msgs:
        print(msgs, file=sys.stderr)
    return obj


def build(force: bool = True, extra_flags=(), output: str = None) -> str:
    """Compile every csrc/*.hip for gfx950 and link liblvx.so; returns its path.  With `output`
    the library goes to that path instead (a variant built with other definitions, to be loaded
    through the LVX_LIB environment variable), its objects into a directory of their own."""
    global OBJ
    lib, obj_dir = LIB, OBJ
    if output:
        lib = os.path.abspath(output)
        OBJ = os.path.join(obj_dir, "variant_" + os.path.basename(lib).replace(".", "_"))
    try:
        os.makedirs(OBJ, exist_ok=True)
        srcs = sorted(glob.glob(os.path.join(CSRC, "*.hip")))
        with ThreadPoolExecutor(max_workers=min(8, len(srcs))) as ex:
            objs = list(ex.map(lambda s: _compile(s, force, extra_flags), srcs))
    finally:
        OBJ = obj_dir
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib] + objs
    subprocess.run(cmd, check=True)
    return lib


if __name__ == "__main__":
    # --define NAME=VALUE (repeatable): extra preprocessor definitions, e.g. the measurement switches
    # of the fused backward kernel
    # --output PATH: link the library there instead of replacing liblvx.so
    defs = [f"-D{sys.argv[i + 1]}" for i, a in enumerate(sys.argv[:-1]) if a == "--define"]
    outs = [sys.argv[i + 1] for i, a in enumerate(sys.argv[:-1]) if a == "--output"]
    print(build(force="--incremental" not in sys.argv or bool(defs), extra_flags=defs,
                output=outs[-1] if outs else None))
