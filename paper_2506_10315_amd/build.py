"""Build liblopt.so (HIP, gfx950) in-tree with hipcc. `python -m paper_2506_10315_amd.build`."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OUT = os.path.join(PKG, "liblopt.so")
OBJ = os.path.join(PKG, "_build")

# (source, object suffix, extra defines): the apply pass is compiled once per optimizer kind
UNITS = [
    ("lopt_api.hip", "api", []),
    ("lopt_kernels.hip", "kernels", []),
    ("lopt_apply_valu.hip", "apply_small_fc", ["-DLOPT_APPLY_KIND=0"]),
    ("lopt_apply_valu.hip", "apply_velo", ["-DLOPT_APPLY_KIND=1"]),
    ("lopt_apply_mfma.hip", "apply_mfma", []),
    ("lopt_apply_f16s.hip", "apply_f16s", []),
    ("lopt_apply_velo4.hip", "apply_velo4", []),
]

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         # packed FP32 instructions are kept out of every kernel
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]


def _run(cmd):
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in p.stdout.splitlines() if "packed-fp32-ops" not in l)
    if p.returncode != 0:
        raise RuntimeError("command failed: %s\n%s" % (" ".join(cmd), out))
    return out


def build(verbose: bool = False, jobs: int = 6, out: str = OUT, extra_defs=(), obj_dir: str = OBJ) -> str:
    """Compile every translation unit (in parallel) and link liblopt.so. `out`, `extra_defs` and `obj_dir`
    exist for A/B builds of experimental variants; the product build uses the defaults."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(obj_dir, exist_ok=True)
    objs = []
    cmds = []
    for src, tag, defs in UNITS:
        o = os.path.join(obj_dir, tag + ".o")
        objs.append(o)
        cmds.append([hipcc, *FLAGS, *defs, *extra_defs, "-c", os.path.join(CSRC, src), "-o", o])
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        for log in ex.map(_run, cmds):
            if verbose and log.strip():
                print(log)
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", out])
    return out


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
