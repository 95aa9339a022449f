"""Build libatk.so (HIP, gfx950) in-tree with hipcc.

    python -m paper_2506_04165_amd.build [--force]

Each source is compiled to an object in parallel, then linked.  hipcc
cross-compiles, so no GPU is needed to build.
"""
from __future__ import annotations

import concurrent.futures
import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libatk.so")
ARCH = "gfx950"

SOURCES = [
    "api.hip",
    "topk_exact.hip",
    "certify.hip",
    "approx_finish.hip",
    "mips_fused.hip",
    "mips_fused_long.hip",
    "valu_probe.hip",
    "read_probe.hip",
    "approx_inst_f32_small.hip",
    "approx_inst_f32_wide.hip",
    "approx_inst_bf16_small.hip",
    "approx_inst_bf16_wide.hip",
    "approx_inst_f32_unaligned.hip",
    "approx_inst_bf16_unaligned.hip",
    "approx_inst_bf16_packed.hip",
    "approx_inst_batched.hip",
    "approx_inst_f32_defer.hip",
    "approx_inst_bf16_defer.hip",
    "approx_inst_bf16_long.hip",
    "approx_inst_i32_small.hip",
    "approx_inst_i32_wide.hip",
    "approx_inst_i32_unaligned.hip",
    "approx_inst_u32_small.hip",
    "approx_inst_u32_wide.hip",
    "approx_inst_u32_unaligned.hip",
    "recall.cpp",
    "select_params.cpp",
]

# packed fp32 instructions are disabled on purpose (they have misbehaved on the test machines)
HIP_FLAGS = ["-O3", "-std=c++17", "-fPIC", f"--offload-arch={ARCH}", "-Wall", "-Wno-unused-function",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


# Per-source additions.  The fused inner-product kernel consumes every matrix result with the
# vector ALU at once: keeping the results in ordinary VGPRs saves one move per score.
FILE_FLAGS = {
    "mips_fused.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"],
}


def _headers_mtime() -> float:
    paths = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    paths.append(os.path.join(os.path.dirname(PKG), "include", "atk.h"))
    return max(os.path.getmtime(p) for p in paths)


def _compile(src: str, force: bool, extra=(), objdir: str = OBJ) -> str:
    path = os.path.join(CSRC, src)
    obj = os.path.join(objdir, src.rsplit(".", 1)[0] + ".o")
    stale = (force or not os.path.exists(obj)
             or os.path.getmtime(obj) < max(os.path.getmtime(path), _headers_mtime()))
    if stale:
        cmd = (["hipcc"] + HIP_FLAGS + FILE_FLAGS.get(src, []) + list(extra)
               + (["-x", "hip"] if src.endswith(".hip") else [])
               + ["-c", path, "-o", obj])
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{r.stdout}\n{r.stderr}")
        noise = "'-packed-fp32-ops' is not a recognized feature"
        err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
        if err.strip():
            sys.stderr.write(err + "\n")
    return obj


def build(force: bool = False, jobs: int | None = None, extra=(), out: str = LIB) -> str:
    """Compile and link.  `extra` adds compiler flags (e.g. -D switches for an experiment) and
    `out` names the library to write; the default is the product library."""
    objdir = OBJ if out == LIB else OBJ + "_" + os.path.basename(out).replace(".", "_")
    os.makedirs(objdir, exist_ok=True)
    jobs = jobs or min(8, os.cpu_count() or 1)
    with concurrent.futures.ThreadPoolExecutor(jobs) as ex:
        objs = list(ex.map(lambda s: _compile(s, force, extra, objdir), SOURCES))
    if force or not os.path.exists(out) or any(os.path.getmtime(o) > os.path.getmtime(out) for o in objs):
        cmd = ["hipcc", "-shared", "-fPIC", f"--offload-arch={ARCH}", "-o", out] + objs
        subprocess.run(cmd, check=True)
    return out


if __name__ == "__main__":
    args = [a for a in sys.argv[1:] if a != "--force"]
    out = LIB
    extra = []
    for a in args:
        if a.startswith("--out="):
            out = os.path.abspath(a[6:])
        else:
            extra.append(a)
    print(build(force="--force" in sys.argv, extra=extra, out=out))
