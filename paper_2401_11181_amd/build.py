"""Build libtetri.so (HIP, gfx950 only) in-tree with hipcc."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libtetri.so")
SOURCES = ["tetri_host.cpp", "tetri_plan.cpp", "tetri_append.hip", "tetri_kv_transfer.hip", "tetri_decode.hip", "tetri_attn.hip"]
HEADERS = [os.path.join(CSRC, "tetri_internal.h"), os.path.join(CSRC, "tetri_plan.h"), os.path.join(CSRC, "attn_common.h"), os.path.join(ROOT, "include", "tetri.h")]

# packed-fp32 instructions are switched off for all device code
HIP_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-Wno-unused-command-line-argument", "-Wno-ignored-attributes"]


def hipcc():
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def build(force=True, verbose=False, extra_flags=()):
    """Compile every source and link libtetri.so.  Returns its path."""
    objs = []
    for src in SOURCES:
        path = os.path.join(CSRC, src)
        obj = os.path.join(CSRC, os.path.splitext(src)[0] + ".o")
        deps = [path] + HEADERS
        if force or not os.path.exists(obj) or any(os.path.getmtime(d) > os.path.getmtime(obj) for d in deps):
            cmd = [hipcc(), "-x", "hip", "-c", path, "-o", obj, "-I", os.path.join(ROOT, "include"), "-I", CSRC,
                   "-DTETRI_BUILDING=1"] + HIP_FLAGS + list(extra_flags)
            if verbose:
                print(" ".join(cmd), flush=True)
            res = subprocess.run(cmd, capture_output=True, text=True)
            noise = "is not a recognized feature for this target"
            err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
            if res.returncode != 0:
                raise RuntimeError("hipcc failed for %s:\n%s" % (src, err))
            if err.strip() and verbose:
                print(err, file=sys.stderr)
        objs.append(obj)
    cmd = [hipcc(), "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + objs
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n" + res.stderr)
    return LIB


if __name__ == "__main__":
    print(build(force="--incremental" not in sys.argv, verbose=True))
