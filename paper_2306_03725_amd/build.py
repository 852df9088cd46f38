"""Builds libusl.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
import os
import re
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


def check_untracked_load(verbose=False):
    """k_bwi_lds and k_both_lds warm the L2 with a load issued from inline assembly: the compiler does not know that its result
    arrives later, so no wait is put behind it -- and nothing but the source's own `s_waitcnt vmcnt(0)` at the top of
    the next pass protects the destination register.  That holds as long as the compiler neither reads nor writes that
    register anywhere in the loop (a copy or a spill right behind the load would free it for another value, which the
    late data would then overwrite).  This looks at the compiler's own assembly listing of the file (same flags as the
    build) and fails the build if the register is mentioned anywhere in the loop but in the load itself."""
    src = os.path.join(CSRC, "k_backward_input_lds.hip")
    lst = os.path.join(HERE, "_build", "k_backward_input_lds.s")
    subprocess.check_call([_hipcc()] + FLAGS + ["--cuda-device-only", "-S", src, "-o", lst])
    with open(lst) as fh:
        text = fh.read().splitlines()
    try:
        checked = scan_listing_for_untracked_load(text, lst)
    except RuntimeError:
        os.rename(lst, lst + ".failed")   # so that an incremental build checks again
        raise
    if verbose:
        print("check_untracked_load: %d warm-up load(s) checked, their registers are untouched inside the loop" % checked, flush=True)


def scan_listing_for_untracked_load(lines, lst="listing"):
    """The check itself, on the lines of an assembly listing; returns the number of loads it looked at."""
    start = [i for i, l in enumerate(lines) if re.match(r"^_Z\w*k_(bwi|both)_lds\w*:", l)]
    if not start:
        raise RuntimeError("check_untracked_load: no k_bwi_lds in the listing")
    checked = 0
    for f0 in start:
        f1 = next(i for i in range(f0, len(lines)) if lines[i].startswith(".Lfunc_end"))
        # basic blocks: (first line, last line, text of the label / comment lines that head the block)
        heads = [i for i in range(f0, f1) if re.match(r"^(\.LBB\d+_\d+:|; %bb\.\d+:)", lines[i])]
        blocks = []
        for n, h in enumerate(heads):
            end = heads[n + 1] if n + 1 < len(heads) else f1
            note, j = lines[h], h + 1
            while j < end and lines[j].lstrip().startswith(";") and "ASM" not in lines[j]:
                note += " " + lines[j]
                j += 1
            blocks.append((h, end, note))
        loads = [i for i in range(f0, f1) if "ASMSTART" in lines[i - 1] and re.search(r"global_load_dword v\d+, (v\d+, s\[|v\[\d+:\d+\], off)", lines[i])]
        if len(loads) < 1:
            raise RuntimeError("check_untracked_load: no warm-up load found in %s" % lines[f0])
        for ld in loads:
            reg = int(re.search(r"global_load_dword v(\d+),", lines[ld]).group(1))
            mine = next(b for b in blocks if b[0] <= ld < b[1])
            m_ = re.search(r"Header=(BB\d+_\d+) Depth=(\d+)", mine[2])
            if not m_:
                raise RuntimeError("check_untracked_load: the warm-up load is not inside a loop")
            header = m_.group(1)
            if m_.group(2) != "1":   # in a loop inside the loop over the passes: the outermost one is meant
                inner = next(b for b in blocks if lines[b[0]].startswith("." + "L" + header + ":"))
                m_ = re.search(r"Parent Loop (BB\d+_\d+) Depth=1", inner[2])
                if not m_:
                    raise RuntimeError("check_untracked_load: no outermost loop found around the warm-up load")
                header = m_.group(1)
            # the loop's blocks: from its header to the last block that names it (loops are laid out in one piece)
            first = next(b[0] for b in blocks if lines[b[0]].startswith("." + "L" + header + ":"))
            last = max(b[1] for b in blocks if ("Header=%s " % header) in b[2] + " " or ("Parent Loop %s " % header) in b[2] + " ")
            in_loop = [b for b in blocks if first <= b[0] < last]

            def mentions(text):
                if re.search(r"\bv%d\b" % reg, text):
                    return True
                return any(int(a) <= reg <= int(b) for a, b in re.findall(r"\bv\[(\d+):(\d+)\]", text))
            reloads = []
            for b0, b1, _ in in_loop:
                for i in range(b0, b1):
                    code = lines[i].split(";")[0]
                    if i != ld and mentions(code):
                        raise RuntimeError("check_untracked_load: v%d, which receives the warm-up load of k_bwi_lds, is also used at "
                                           "%s:%d: %s" % (reg, lst, i + 1, lines[i].strip()))
                    if "scratch_load" in code:
                        reloads.append(i + 1)
            # The kernel lives at the edge of a lane's 128 registers.  One reload in the loop is known and harmless (the lane
            # number, in the branch for overflow lists that LDS cannot hold); any other sits among the gathers, where its
            # wait also waits for the warm-up load: 0.15 ms per call at m = 500k, 0.8 ms at the bf16 benchmark shape.
            if len(reloads) > 1:
                raise RuntimeError("check_untracked_load: %d register reloads inside the loop of k_bwi_lds (%s lines %s): the "
                                   "kernel needs more registers than a lane has" % (len(reloads), lst, reloads))
            checked += 1
    return checked


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
    lds_src, lds_lst = os.path.join(CSRC, "k_backward_input_lds.hip"), os.path.join(HERE, "_build", "k_backward_input_lds.s")
    if force or not os.path.exists(lds_lst) or os.path.getmtime(lds_lst) < max(os.path.getmtime(lds_src), newest_dep):
        check_untracked_load(verbose)
    subprocess.check_call([_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs)
    csrc = os.path.join(CSRC, "ceilings.hip")
    if force or not os.path.exists(LIB_CEILINGS) or os.path.getmtime(LIB_CEILINGS) < os.path.getmtime(csrc):
        subprocess.check_call([_hipcc()] + FLAGS + ["-shared", csrc, "-o", LIB_CEILINGS])
    return LIB


if __name__ == "__main__":
    print(build(force="--incremental" not in sys.argv, verbose=True))
