"""Builds libfate.so (HIP, gfx950) in-tree with hipcc."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libfate.so")
SOURCES = ["api.cpp", "route.hip", "pack.hip", "ffn.hip", "ffn_decode.hip", "layer_decode.hip", "layer_decode_b1.hip", "layer_decode_loop_r41.hip", "layer_decode_loop_r42.hip", "layer_decode_loop_r44.hip", "layer_decode_loop_r82.hip", "layer_decode_loop_r84.hip", "ffn_prefill.hip", "cache.cpp",
           "cache_hip.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang",
         "-packed-fp32-ops", "-Wno-unused-result", "-Wno-unknown-warning-option"]


def _newest_header():
    hdrs = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    hdrs += [os.path.join(HERE, "..", "include", f) for f in os.listdir(os.path.join(HERE, "..", "include"))]
    return max(os.path.getmtime(h) for h in hdrs)


def _compile(src, objdir):
    path = os.path.join(CSRC, src)
    obj = os.path.join(objdir, src + ".o")
    # FATE_INCREMENTAL=1 (development only): keep objects newer than their source and every header
    if os.environ.get("FATE_INCREMENTAL") and os.path.exists(obj) and \
            os.path.getmtime(obj) > max(os.path.getmtime(path), _newest_header()):
        return src, obj, 0, ""
    cmd = [HIPCC, *FLAGS, "-x", "hip", "-c", path, "-o", obj]
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in p.stdout.splitlines() if "packed-fp32-ops" not in l)
    return src, obj, p.returncode, out


def build(verbose=True, jobs=8):
    """Compiles every source (the long ones first, `jobs` at a time) and links libfate.so."""
    from concurrent.futures import ThreadPoolExecutor
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    srcs = [s for s in SOURCES if os.path.exists(os.path.join(CSRC, s))]
    order = sorted(srcs, key=lambda s: (not s.startswith("layer_decode"), s != "ffn_prefill.hip", srcs.index(s)))
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        results = list(pool.map(lambda s: _compile(s, objdir), order))
    objs = {}
    for src, obj, rc, out in results:
        if rc != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{out}")
        if verbose and out.strip():
            print(f"[{src}]\n{out}")
        objs[src] = obj
    cmd = [HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB, *[objs[s] for s in srcs]]
    out = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if out.returncode != 0:
        raise RuntimeError("link failed:\n" + out.stdout)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build()
