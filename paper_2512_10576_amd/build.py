"""Build libess.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree.

    python -m paper_2512_10576_amd.build

Objects go to `_build/` (ignored by git); the library lands next to this
file so that it travels with the source tree.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OUT = os.path.join(HERE, "libess.so")
SOURCES = ["ess_api.hip", "index_score.hip", "index_select.hip", "index_sample.hip", "topk.hip", "cache.hip", "sparse_mla.hip"]
FLAGS = ["-O3", "--offload-arch=gfx950", "-fPIC", "-std=c++17", "-I" + os.path.join(ROOT, "include"),
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]


# per-source additions: sparse_mla.hip keeps the results of compiler-generated MFMAs in VGPRs, because its
# kernel holds the output accumulators in AGPRs that it names itself (see the comment there)
EXTRA_FLAGS = {"sparse_mla.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form", "-std=c++20"]}


def compile_flags(src: str) -> list:
    extra = EXTRA_FLAGS.get(src, [])
    base = [f for f in FLAGS if not (f.startswith("-std=") and any(e.startswith("-std=") for e in extra))]
    return [*base, *extra]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def _run(cmd):
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    keep = [l for l in p.stdout.splitlines() if "packed-fp32-ops" not in l]
    if p.returncode != 0:
        raise RuntimeError("command failed: %s\n%s" % (" ".join(cmd), "\n".join(keep)))
    return "\n".join(keep)


def build(verbose: bool = False) -> str:
    """Compile every source and link the shared library; returns its path."""
    hipcc = _hipcc()
    bdir = os.path.join(ROOT, "_build")
    os.makedirs(bdir, exist_ok=True)
    objs = [os.path.join(bdir, s.replace(".hip", ".o")) for s in SOURCES]

    def one(pair):
        src, obj = pair
        return _run([hipcc, *compile_flags(src), "-c", os.path.join(CSRC, src), "-o", obj])

    with ThreadPoolExecutor(max_workers=min(6, len(SOURCES))) as ex:
        logs = list(ex.map(one, zip(SOURCES, objs)))
    logs.append(_run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", OUT]))
    if verbose:
        print("\n".join(l for l in logs if l))
    return OUT


if __name__ == "__main__":
    print(build(verbose=True))
