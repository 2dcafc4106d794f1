"""Builds libredist.so in-tree: host C++ (planner, C-ABI) + gfx950 HIP kernels."""
import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libredist.so")
HOST_SOURCES = ["planner.cpp", "copyop.cpp", "cellop.cpp", "api.cpp"]
HIP_SOURCES = ["kernels.hip"]
# packed fp32 instruction selection is switched off for all device code on the test machines
DEVICE_FLAGS = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _run(cmd):
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if proc.returncode != 0:
        sys.stderr.write(proc.stdout)
        raise RuntimeError("command failed: " + " ".join(cmd))
    return proc.stdout


def build(verbose=False):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    obj_dir = os.path.join(HERE, "_build")
    os.makedirs(obj_dir, exist_ok=True)
    common = ["-O3", "-std=c++17", "-fPIC", "-Wall", "-I", os.path.join(ROOT, "include"), "-I", CSRC]
    objs = []
    for src in HOST_SOURCES:
        obj = os.path.join(obj_dir, src + ".o")
        _run([hipcc, "-x", "c++", "-D__HIP_PLATFORM_AMD__", "-I", "/opt/rocm/include"] + common +
             ["-c", os.path.join(CSRC, src), "-o", obj])
        objs.append(obj)
    for src in HIP_SOURCES:
        obj = os.path.join(obj_dir, src + ".o")
        out = _run([hipcc, "-x", "hip"] + DEVICE_FLAGS + common + ["-c", os.path.join(CSRC, src), "-o", obj])
        if verbose:
            print(out)
        objs.append(obj)
    _run([hipcc, "-shared", "-fPIC"] + DEVICE_FLAGS + objs + ["-o", LIB])
    return LIB


def build_host_selftest(sanitize=True):
    """Host-only self-test of planner, descriptor builder and plan objects (csrc/host_selftest.cpp), by default with
    AddressSanitizer and UndefinedBehaviorSanitizer.  Host code only: the kernel launchers are stubs, no GPU code is
    compiled or instrumented.  Returns the path of the executable; run it to carry out the test."""
    cxx = shutil.which("g++") or "g++"
    obj_dir = os.path.join(HERE, "_build")
    os.makedirs(obj_dir, exist_ok=True)
    exe = os.path.join(obj_dir, "host_selftest_asan" if sanitize else "host_selftest")
    flags = ["-O1", "-g", "-std=c++17", "-Wall", "-D__HIP_PLATFORM_AMD__", "-I", "/opt/rocm/include",
             "-I", os.path.join(ROOT, "include"), "-I", CSRC]
    if sanitize:
        flags += ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer"]
    srcs = [os.path.join(CSRC, f) for f in HOST_SOURCES + ["host_selftest.cpp"]]
    _run([cxx] + flags + srcs + ["-L", "/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath,/opt/rocm/lib", "-o", exe])
    return exe


if __name__ == "__main__":
    if "--sanitize" in sys.argv:
        exe = build_host_selftest(True)
        print(exe)
        sys.exit(subprocess.call([exe] + [a for a in sys.argv[1:] if a.isdigit()]))
    print(build(verbose=True))
