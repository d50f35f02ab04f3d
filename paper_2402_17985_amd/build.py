"""Build libfq.so (the HIP kernels and the C-ABI layer) for gfx950 with hipcc, in-tree."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OUT = os.path.join(HERE, "libfq.so")
# (source, extra flags, object name); fq_gemm.hip is built once per operand mode, in parallel
SOURCES = [("fq_gemm.hip", ["-DFQ_GEMM_MODE=1"], "fq_gemm_i4.o"),
           ("fq_gemm.hip", ["-DFQ_GEMM_MODE=0"], "fq_gemm_i8.o"),
           ("fq_gemm.hip", ["-DFQ_GEMM_MODE=2"], "fq_gemm_bf16.o"),
           ("fq_gemm.hip", ["-DFQ_GEMM_MODE=3"], "fq_gemm_f6.o"),
           ("fq_api.hip", [], "fq_api.o"), ("fq_quant.hip", [], "fq_quant.o"),
           ("fq_gemm_select.hip", [], "fq_gemm_select.o"), ("fq_peak.hip", [], "fq_peak.o")]
# -packed-fp32-ops off: keeps the compiler from forming packed fp32 instructions
# -ffp-contract=off: every fp32 multiply stays a single correctly rounded operation
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function", "-Wno-unknown-attributes"]


def _hipcc():
    for c in ("/opt/rocm/bin/hipcc", "hipcc"):
        if os.path.isabs(c) and os.path.exists(c):
            return c
    return "hipcc"


def _newer(target, deps):
    if not os.path.exists(target):
        return False
    t = os.path.getmtime(target)
    return all(os.path.getmtime(d) <= t for d in deps)


def build(force: bool = True, verbose: bool = False) -> str:
    hdrs = [os.path.join(CSRC, "fq_internal.h"), os.path.join(HERE, "..", "include", "fq.h"),
            os.path.join(HERE, "..", "include", "fq_peak.h")]
    srcs = [(os.path.join(CSRC, s), extra, obj) for s, extra, obj in SOURCES]
    if not force and _newer(OUT, [s for s, _, _ in srcs] + hdrs):
        return OUT                          # nothing changed since the library was linked
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    hipcc = _hipcc()

    def compile_one(item):
        src, extra, objname = item
        obj = os.path.join(objdir, objname)
        if not force and _newer(obj, [src] + hdrs):
            return obj                      # incremental build: this object is up to date
        cmd = [hipcc] + FLAGS + extra + ["-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed for {src}:\n{r.stdout}\n{r.stderr}")
        return obj

    with ThreadPoolExecutor(max_workers=len(srcs)) as ex:
        objs = list(ex.map(compile_one, srcs))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", OUT] + objs
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")
    return OUT


if __name__ == "__main__":
    # `python -m paper_2402_17985_amd.build` rebuilds everything; `... build --changed` only what changed
    print(build(force="--changed" not in sys.argv, verbose=True))
    sys.exit(0)
