"""Builds libie_attn.so (the C-ABI library) for gfx950 with hipcc, in-tree."""
import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libie_attn.so")
SOURCES = ["ie_attn_api.hip", "attn_fwd.hip", "attn_fwd_wide.hip", "attn_bwd.hip", "sp_permute.hip", "linear_gemm.hip"]
# -fno-honor-nans: the kernels never produce NaN from finite inputs (masked scores are -inf and only ever
# meet finite references), and without it every max is preceded by a canonicalising self-max.
# Packed fp32 VALU forms are switched off for all device code (known to misbehave on the test machines).
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang",
         "-packed-fp32-ops", "-fno-honor-nans", "-Wall", "-Wno-unused-command-line-argument",
         "-Rpass-analysis=kernel-resource-usage"]
# Kernels that load operands into AGPRs from assembly (the compiler does not know these are
# loads, so a spill of such a register right after the statement would save it before the data
# has arrived) and keep ~450 registers live: they must compile without scratch.  The recomputing dQ
# kernel is listed because a spill in it has only ever meant a per-item invariant hoisted out of the
# item loop, which is cheaper to recompute.
NO_SCRATCH = ("attn_fwd_wide_kernel", "attn_bwd_dkdv_kernelILi128E", "attn_bwd_dq_kernelILi128E")
# Persistent kernels loop over work items around a body that leaves no register free: with machine LICM the
# compiler hoists per-lane invariants of the item prologue out of that loop and spills to keep them.
SOURCE_FLAGS = {"attn_fwd_wide.hip": ["-mllvm", "-disable-machine-licm"], "attn_bwd.hip": ["-mllvm", "-disable-machine-licm"]}


def _check_scratch(src, remarks):
    name = None
    for line in remarks.splitlines():
        if "Function Name:" in line:
            name = line.split("Function Name:")[1].split()[0]
        elif "ScratchSize [bytes/lane]:" in line and name:
            size = int(line.split("ScratchSize [bytes/lane]:")[1].split()[0])
            if size and any(k in name for k in NO_SCRATCH):
                raise RuntimeError(f"{src}: {name} spills to scratch ({size} bytes/lane); see NO_SCRATCH in build.py")


def _compile(src, extra, objdir=CSRC):
    obj = os.path.join(objdir, src.replace(".hip", ".o"))
    cmd = ["hipcc", *FLAGS, *SOURCE_FLAGS.get(src, []), *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    lines = [l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l]
    remarks = "\n".join(l for l in lines if "remark:" in l)
    context = re.compile(r"^\s*\d*\s*\|")   # source excerpts under a diagnostic
    err = "\n".join(l for l in lines if "remark:" not in l and not context.match(l))
    if r.returncode == 0 and "warning" not in err:   # only the include trail of a remark is left
        err = ""
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{err}")
    _check_scratch(src, remarks)
    return obj, err


def build_variant(name, extra):
    """The library with extra compile flags (instrumented or what-if builds), as
    _variants/libie_attn_<name>.so next to the real one; select it with IE_ATTN_LIB."""
    vdir = os.path.join(HERE, "_variants")
    odir = os.path.join(vdir, "obj_" + name)
    os.makedirs(odir, exist_ok=True)
    with ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        objs = [o for o, _ in ex.map(lambda s: _compile(s, list(extra), odir), SOURCES)]
    lib = os.path.join(vdir, f"libie_attn_{name}.so")
    r = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    return lib


def build(verbose=False, extra=()):
    with ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        results = list(ex.map(lambda s: _compile(s, list(extra)), SOURCES))
    objs = [o for o, _ in results]
    if verbose:
        for _, err in results:
            if err.strip():
                print(err, file=sys.stderr)
    r = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    # A kernel whose host stub was not emitted shows up only as a lazily bound undefined symbol.
    r = subprocess.run(["nm", "-D", "--undefined-only", LIB], capture_output=True, text=True)
    missing = [l.split()[-1] for l in r.stdout.splitlines() if "_ZN2ie" in l]
    if missing:
        raise RuntimeError("libie_attn.so has undefined symbols of its own namespace: " + ", ".join(missing))
    return LIB


if __name__ == "__main__":
    print(build(verbose=True, extra=sys.argv[1:]))
