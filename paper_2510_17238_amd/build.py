"""Compile the HIP sources under csrc/ for gfx950 (explicit hipcc, in-tree): libst.so, the library of the path, and
libst_probe.so, the machine probes of the benchmark (a library of their own: the path does not need them)."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libst.so")
PROBE_LIB = os.path.join(HERE, "libst_probe.so")

SOURCES = ["st_error.hip", "st_rope.hip", "st_plan.hip", "st_prefill.hip", "st_prefill_bwd.hip", "st_cache.hip", "st_decode.hip", "st_sched.hip"]
PROBE_SOURCES = ["st_probe.hip"]            # (linked with st_error.o for the error text)

FLAGS = [
    "--offload-arch=gfx950:xnack-", "-O3", "-std=c++17", "-fPIC",
    # keep the compiler from forming packed-fp32 VALU ops
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
]


# per-file extras.  The backward kernels run one wave per SIMD and keep their big accumulators in place; with
# the matrix instructions writing ordinary vector registers the compiler stops shuttling score blocks
# through the accumulation registers (12 % on the query-side kernel).  The forward file manages its
# accumulation registers by hand and must not get this.
EXTRA_FLAGS = {"st_prefill_bwd.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"]}


def _hipcc():
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def build_library(verbose=True):
    """Always recompiles every source; returns the path of the shared library."""
    os.makedirs(BUILD, exist_ok=True)
    hipcc = _hipcc()
    objs = []
    procs = []
    for src in SOURCES + PROBE_SOURCES:
        obj = os.path.join(BUILD, src.replace(".hip", ".o"))
        cmd = [hipcc] + FLAGS + EXTRA_FLAGS.get(src, []) + ["-c", os.path.join(CSRC, src), "-o", obj]
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    for src, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{out}")
        if verbose and out.strip():
            print(out)
    n_main = len(SOURCES)
    for lib, members in ((LIB, objs[:n_main]), (PROBE_LIB, objs[n_main:] + [objs[SOURCES.index("st_error.hip")]])):
        cmd = [hipcc, "--offload-arch=gfx950:xnack-", "-shared", "-fPIC", "-o", lib] + members
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if r.returncode != 0:
            raise RuntimeError("link failed:\n" + r.stdout)
        if verbose:
            print("built", lib)
    return LIB


if __name__ == "__main__":
    build_library()
    sys.exit(0)
