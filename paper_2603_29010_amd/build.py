"""Build libucl.so: every HIP translation unit compiled for gfx950 with hipcc, in parallel, in-tree.

Run as ``python -m paper_2603_29010_amd.build`` (or call ``build()``).  Object files and the
library stay inside the package directory; nothing is installed.
"""
import concurrent.futures
import glob
import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(CSRC, "_build")
LIB = os.path.join(HERE, "libucl.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-mllvm", "-disable-promote-alloca-to-lds",
         "-Wno-pass-failed", "-Wno-unused-variable", "-Wno-unused-but-set-variable"]


def _compile(src, force):
    obj = os.path.join(OBJ, os.path.basename(src) + ".o")
    deps = [src] + glob.glob(os.path.join(CSRC, "*.h")) + [os.path.join(HERE, "..", "include", "ucl.h")]
    if not force and os.path.exists(obj) and os.path.getmtime(obj) >= max(os.path.getmtime(d) for d in deps):
        return obj, ""
    cmd = [HIPCC] + FLAGS + ["-save-temps=obj", "-c", src, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True, cwd=OBJ)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{r.stderr}")
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    _check_asm(obj)
    return obj, err


def _check_asm(obj):
    """Refuse kernels that spill to scratch: accumulators must live in registers."""
    stem = os.path.basename(obj)[:-len(".hip.o")]
    for asm in glob.glob(os.path.join(OBJ, stem + "-hip-amdgcn-amd-amdhsa-gfx950.s")):
        text = open(asm).read()
        names = re.findall(r"\.amdhsa_kernel\s+(\S+)", text)
        sizes = re.findall(r"\.amdhsa_private_segment_fixed_size\s+(\d+)", text)
        if len(names) != len(sizes):
            raise RuntimeError(f"{asm}: cannot match kernels to their scratch sizes")
        for name, scratch in zip(names, sizes):
            if int(scratch) != 0:
                raise RuntimeError(f"kernel {name} uses {scratch} bytes of scratch memory")
        if re.search(r"s_swappc_b64", text):
            raise RuntimeError(f"{asm}: a kernel calls a function (a loop body was not inlined)")
        # A buffer resource that the register allocator moved into vector registers (the tile kernels sit at their
        # scalar-register budget) makes every global -> LDS copy a readfirstlane loop: 14 % slower when it happened.
        lines = text.split("\n")
        for k, line in enumerate(lines):
            if "buffer_load_dword" in line and line.rstrip().endswith(" lds") and \
                    any("v_readfirstlane_b32" in x for x in lines[max(0, k - 10):k]) and \
                    any("s_cbranch_execnz" in x for x in lines[k + 1:k + 6]):
                raise RuntimeError(f"{asm}: line {k + 1}: a global -> LDS copy sits in a readfirstlane loop "
                                   "(its buffer resource is held in vector registers)")


def build(force=False, jobs=None, verbose=False):
    os.makedirs(OBJ, exist_ok=True)
    srcs = sorted(glob.glob(os.path.join(CSRC, "*.hip")))
    jobs = jobs or min(8, os.cpu_count() or 1)
    objs = []
    with concurrent.futures.ThreadPoolExecutor(jobs) as ex:
        for obj, err in ex.map(lambda s: _compile(s, force), srcs):
            objs.append(obj)
            if verbose and err.strip():
                print(err, file=sys.stderr)
    newest = max(os.path.getmtime(o) for o in objs)
    if force or not os.path.exists(LIB) or os.path.getmtime(LIB) < newest:
        subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv, verbose=True))
