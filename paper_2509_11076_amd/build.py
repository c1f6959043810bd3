"""Build libss.so (the HIP library behind the C ABI of include/ss.h) in-tree for gfx950."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SOURCES = ["ss_runtime.hip", "ss_copy.hip", "ss_trace.hip", "ss_scan.hip", "ss_match.hip", "ss_policy.hip", "ss_generator.hip", "ss_align.hip"]
LIB = os.path.join(HERE, "libss.so")


def build_library(verbose=True):
    """Compile every HIP source for gfx950 and link the shared library.  Always recompiles."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    bdir = os.path.join(HERE, "_build")
    os.makedirs(bdir, exist_ok=True)
    common = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
              "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
              "-Wall", "-Wno-unused-function", "-Wno-unused-command-line-argument",
              "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(HERE, "csrc")]
    procs = []
    for src in SOURCES:
        obj = os.path.join(bdir, src.replace(".hip", ".o"))
        objs.append(obj)
        cmd = common + ["-c", os.path.join(HERE, "csrc", src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    for src, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l and l.strip())
        if p.returncode != 0:
            raise RuntimeError("hipcc failed on %s:\n%s" % (src, out))
        if verbose and out:
            print(out, flush=True)
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


HOOK_LIB = os.path.join(HERE, "libss_torch_hook.so")


def build_hook(verbose=True):
    """Compile the PyTorch dispatch hook (host C++ only) against the installed PyTorch and libss.so."""
    import sysconfig
    import torch
    from torch.utils import cpp_extension as ce
    tlib = os.path.join(os.path.dirname(torch.__file__), "lib")
    cmd = ["g++", "-O2", "-std=c++17", "-fPIC", "-shared", "-Wall", "-Wno-unused-function",
           "-D__HIP_PLATFORM_AMD__=1", "-DUSE_ROCM=1",
           "-DNDEBUG",      # as PyTorch's own build: its inline debug checks read members a release build never sets
           "-D_GLIBCXX_USE_CXX11_ABI=%d" % int(torch._C._GLIBCXX_USE_CXX11_ABI)]
    cmd += ["-I" + p for p in ce.include_paths()]
    cmd += ["-I/opt/rocm/include", "-I" + sysconfig.get_paths()["include"],
            "-I" + os.path.join(ROOT, "include"), os.path.join(HERE, "csrc", "ss_torch_hook.cpp"),
            "-o", HOOK_LIB, "-L" + tlib, "-L" + HERE, "-ltorch_cpu", "-lc10", "-lc10_hip", "-lss",
            "-Wl,-rpath,$ORIGIN", "-Wl,-rpath," + tlib]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return HOOK_LIB


if __name__ == "__main__":
    build_library()
    print("built", LIB)
    build_hook()
    print("built", HOOK_LIB)
