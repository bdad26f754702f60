"""Builds liblsam.so (the C-ABI library) for gfx950 with hipcc, in-tree."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "liblsam.so")
SOURCES = ["lsam_api.hip", "kernels_stream.hip", "kernels_gemm.hip", "kernels_gemm_bf16.hip", "kernels_ce.hip", "kernels_conv.hip",
           "kernels_probe.hip", "lsam_static.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]


def build(verbose=True, jobs=4):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    procs = []
    objs = []
    for src in SOURCES:
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        objs.append(obj)
        cmd = [hipcc] + FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)))
    for src, p in procs:
        out = p.communicate()[0].decode()
        lines = [l for l in out.splitlines() if "packed-fp32-ops" not in l]
        if p.returncode != 0:
            raise RuntimeError("compiling %s failed:\n%s" % (src, "\n".join(lines)))
        if verbose and lines:
            print("\n".join(lines))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


SAN_LIB = os.path.join(HERE, "liblsam_san.so")
SAN_FLAGS = ["-Xarch_host", "-fsanitize=address,undefined", "-Xarch_host", "-fno-sanitize-recover=undefined"]


def build_host_sanitized(verbose=True):
    """liblsam_san.so: the same sources with AddressSanitizer and UndefinedBehaviorSanitizer on the
    host code only (the device code is compiled as always; sanitizers do not run on the GPU).
    For checking the host side of the library -- configuration checks, layout, schedule, argument
    validation -- in a process that preloads the ASan runtime; see tests/test_host_sanitizers.py."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "_build", "san")
    os.makedirs(objdir, exist_ok=True)
    procs, objs = [], []
    for src in SOURCES:
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        objs.append(obj)
        flags = [f if f != "-O3" else "-O1" for f in FLAGS] + ["-g"] + SAN_FLAGS
        procs.append((src, subprocess.Popen([hipcc] + flags + ["-c", os.path.join(CSRC, src), "-o", obj],
                                            stdout=subprocess.PIPE, stderr=subprocess.STDOUT)))
    for src, p in procs:
        out = p.communicate()[0].decode()
        if p.returncode != 0:
            raise RuntimeError("compiling %s failed:\n%s" % (src, out))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address,undefined", "-shared-libsan",
           "-o", SAN_LIB] + objs
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return SAN_LIB


def asan_runtime():
    """Path of the shared AddressSanitizer runtime of the ROCm clang, or None."""
    import glob
    hits = glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so")
    return hits[0] if hits else None


if __name__ == "__main__":
    if "--host-sanitizers" in sys.argv[1:]:
        print("built", build_host_sanitized())
    else:
        build()
        print("built", LIB)
