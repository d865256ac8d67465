"""Builds libadapt_fxp.so for gfx950 with hipcc (in-tree, next to this file)."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libadapt_fxp.so")
SOURCES = ["api.hip", "quantize.hip", "kld.hip", "contract_gemm.hip", "contract_fwd.hip",
           "contract_dgrad.hip", "contract_dgrad_s2.hip", "contract_wgrad.hip", "pushup.hip", "sgd.hip",
           "contract_backward.hip", "contract_pair_d64x64.hip", "contract_pair_d128x64.hip", "contract_pair_d64x128.hip",
           "contract_pair_d128x128.hip", "perf_model.hip", "net.hip", "workspace.hip", "bn.hip", "wide.hip", "wide_ops.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-fno-gpu-flush-denormals-to-zero", "-Wall", "-Wno-unused-function",
         # the accumulator loops of the contraction epilogue must be fully unrolled (register arrays)
         "-mllvm", "-pragma-unroll-threshold=262144"]
OBJDIR = os.path.join(HERE, "_build")


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)


def build(verbose: bool = False, only=None, extra_flags=(), lib=LIB, objdir=OBJDIR) -> str:
    """Compiles every source to an object (in parallel) and links the shared library.
    `only` restricts recompilation to the named sources plus whatever is out of date."""
    from concurrent.futures import ThreadPoolExecutor
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(objdir, exist_ok=True)
    inc = ["-I", os.path.join(ROOT, "include"), "-I", CSRC]
    objs = [os.path.join(objdir, s.replace(".hip", ".o")) for s in SOURCES]
    # an object older than its source or than any header is rebuilt even when `only` does not name it: the
    # structs that cross translation units (kernel arguments, plans) must have one layout in the whole library
    headers = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hpp")]
    headers += [os.path.join(ROOT, "include", f) for f in os.listdir(os.path.join(ROOT, "include")) if f.endswith(".h")]
    newest_header = max(os.path.getmtime(h) for h in headers)

    def stale(src, obj):
        return not os.path.exists(obj) or os.path.getmtime(obj) < max(os.path.getmtime(os.path.join(CSRC, src)), newest_header)
    jobs = [(s, o) for s, o in zip(SOURCES, objs) if only is None or s in only or stale(s, o)]
    with ThreadPoolExecutor(max_workers=min(8, max(1, len(jobs)))) as ex:
        list(ex.map(lambda so: _run([hipcc, *FLAGS, *extra_flags, *inc, "-c", os.path.join(CSRC, so[0]), "-o", so[1]], verbose), jobs))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs], verbose)
    return lib


if __name__ == "__main__":
    import sys
    print(build(verbose=True, only=sys.argv[1:] or None))
