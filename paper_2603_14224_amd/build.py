"""Compile the gfx950 HIP sources into paper_2603_14224_amd/libsik.so (in-tree)."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsik.so")
SOURCES = ["sik_api.hip", "sik_quantize.hip", "sik_score.hip", "sik_topk.hip", "sik_attn.hip", "sik_fused.hip", "sik_kvq.hip", "sik_step.hip", "sik_step_bf16.hip", "sik_step_f16.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-munsafe-fp-atomics",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wno-unused-function",
         # the first kernel arguments arrive in scalar registers with the wavefront instead of through a load
         "-mllvm", "-amdgpu-kernarg-preload-count=16"]


def build(verbose: bool = False, defines=(), lib: str = LIB, objdir_name: str = "_build") -> str:
    """Compile every source for gfx950 and link the shared library; `defines` adds -D flags (the
    debug phase-timeline build uses SIK_TIMELINE and another output path)."""
    objdir = os.path.join(HERE, objdir_name)
    os.makedirs(objdir, exist_ok=True)

    def cc(src):
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        cmd = ["hipcc", *FLAGS, *[f"-D{d}" for d in defines], "-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0 or verbose:
            sys.stderr.write(r.stdout + r.stderr)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed on " + src)
        return obj

    with ThreadPoolExecutor(max_workers=min(10, len(SOURCES))) as ex:
        objs = list(ex.map(cc, SOURCES))
    r = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs],
                       capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(r.stdout + r.stderr)
        raise RuntimeError("link failed")
    return lib


if __name__ == "__main__":
    print(build(verbose=True))
