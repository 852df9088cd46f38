"""Builds libusl.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libusl.so")
LIB_CEILINGS = os.path.join(HERE, "libusl_ceilings.so")   # measurement kernels, not part of the training path
SOURCES = ["usl_api.hip", "k_products.hip", "k_elementwise.hip", "k_backward_input.hip",
           "k_redistribute.hip", "k_schedule.hip", "k_predict.hip", "k_sparse_grad.hip", "k_backward_input_lds.hip"]
# -packed-fp32-ops: packed FP32 VALU instructions are switched off (they have produced wrong
# results on the test machines); -munsafe-fp-atomics: hardware float atomic add, no CAS loop.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-munsafe-fp-atomics",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]


def _hipcc():
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def build(force=True, verbose=False):
    objs = []
    procs = []
    os.makedirs(os.path.join(HERE, "_build"), exist_ok=True)
    deps = [os.path.join(CSRC, "usl_internal.h"), os.path.join(CSRC, "k_products_common.h"), os.path.join(HERE, "..", "include", "usl.h")]
    newest_dep = max(os.path.getmtime(p) for p in deps)
    for src in SOURCES:
        sp = os.path.join(CSRC, src)
        obj = os.path.join(HERE, "_build", src.replace(".hip", ".o"))
        objs.append(obj)
        if not force and os.path.exists(obj) and os.path.getmtime(obj) > max(os.path.getmtime(sp), newest_dep):
            continue
        cmd = [_hipcc()] + FLAGS + ["-c", sp, "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    for src, p in procs:
        out, _ = p.communicate()
        if p.returncode != 0:
            sys.stderr.write(out)
            raise RuntimeError("hipcc failed on %s" % src)
    subprocess.check_call([_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs)
    csrc = os.path.join(CSRC, "ceilings.hip")
    if force or not os.path.exists(LIB_CEILINGS) or os.path.getmtime(LIB_CEILINGS) < os.path.getmtime(csrc):
        subprocess.check_call([_hipcc()] + FLAGS + ["-shared", csrc, "-o", LIB_CEILINGS])
    return LIB


if __name__ == "__main__":
    print(build(force="--incremental" not in sys.argv, verbose=True))
