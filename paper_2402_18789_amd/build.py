"""Builds libflexco.so (gfx950) in-tree with hipcc:  `python paper_2402_18789_amd/build.py`
(run as a script, so that the package - which loads the library - is not imported)."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.environ.get("FLEXCO_BUILD_OBJ", os.path.join(ROOT, "_build"))
LIB = os.environ.get("FLEXCO_BUILD_LIB", os.path.join(HERE, "libflexco.so"))
SOURCES = ["flexco_maps.cpp", "flexco_sched.cpp", "flexco_prune.cpp", "flexco_api.hip", "kernels_generic.hip", "attn_generic.hip", "gemm_mfma.hip",
           "attn_mfma.hip", "attn_chunk_mfma.hip", "lora_mfma.hip", "attn_bwd_mfma.hip", "probes.hip", "train_head.hip", "relu_bitmask.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang",
         "-packed-fp32-ops", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC, "-Wno-unused-command-line-argument",
         "-Wno-unknown-warning-option"] + os.environ.get("FLEXCO_BUILD_FLAGS", "").split()


# Per-source flags.  Kernels whose accumulators fit the 256 architectural registers of a wavefront take their matrix
# products in the form that reads and writes plain vector registers: left to its default the compiler parked the
# attention backward's accumulators in accumulation registers and moved them in and out around every product
# (112 moves per step of the dQ kernel beside its 24 products).
SOURCE_FLAGS = {"attn_bwd_mfma.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"]}


def _compile(src):
    obj = os.path.join(OBJ_DIR, os.path.splitext(src)[0] + ".o")
    cmd = [HIPCC, "-x", "hip"] + FLAGS + SOURCE_FLAGS.get(src, []) + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s\n%s" % (src, r.stdout, r.stderr))
    warn = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l and l.strip())
    return obj, warn


def build(verbose=True):
    os.makedirs(OBJ_DIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        results = list(ex.map(_compile, SOURCES))
    objs = [o for o, _ in results]
    if verbose:
        for _, w in results:
            if w:
                print(w, file=sys.stderr)
    # Link against the HIP runtime PyTorch ships (soname libamdhip64.so), so that the library
    # and torch share one runtime, one set of devices and one set of streams in the process.
    import torch
    tlib = os.path.join(os.path.dirname(torch.__file__), "lib")
    cmd = [HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-no-hip-rt", "-o", LIB] + objs + \
          ["-L" + tlib, "-lamdhip64", "-Wl,-rpath," + tlib]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n%s\n%s" % (r.stdout, r.stderr))
    return LIB


HOST_SOURCES = ["flexco_maps.cpp", "flexco_sched.cpp", "flexco_prune.cpp"]


def build_host_sanitized(out_path):
    """The host-only sources (index maps, scheduler, graph pruning) as a library of their own, compiled for the CPU
    with AddressSanitizer and UndefinedBehaviorSanitizer (any finding aborts).  Load it with the sanitizer runtime
    preloaded: LD_PRELOAD=$(g++ -print-file-name=libasan.so) FLEXCO_LIB_PATH=<out_path> FLEXCO_HOST_ONLY=1."""
    cxx = os.environ.get("CXX", "g++")
    cmd = [cxx, "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-shared", "-fPIC", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC] + \
          [os.path.join(CSRC, f) for f in HOST_SOURCES] + ["-o", out_path]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("host sanitized build failed:\n%s\n%s" % (r.stdout, r.stderr))
    return out_path


if __name__ == "__main__":
    if len(sys.argv) > 2 and sys.argv[1] == "--host-sanitized":
        print(build_host_sanitized(sys.argv[2]))
    else:
        print(build())
