"""Build the HIP library (gfx950) in-tree: paper_2506_03700_amd/libadadecode.so, plus the CPU-only
scheduler test hook libad_sched_test.so (host code, g++)."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libadadecode.so")
SCHED_LIB = os.path.join(HERE, "libad_sched_test.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

HIP_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-Wall",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _sources(names):
    return [os.path.join(CSRC, n) for n in names]


def _stale(target, deps):
    if not os.path.exists(target):
        return True
    t = os.path.getmtime(target)
    return any(os.path.getmtime(d) > t for d in deps)


def _all_deps():
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)]
    deps.append(os.path.join(os.path.dirname(HERE), "include", "adadecode.h"))
    return deps


def build_hip(force=True):
    if not force and not _stale(LIB, _all_deps()):
        return LIB
    cmd = [HIPCC] + HIP_FLAGS + ["-o", LIB + ".tmp"] + _sources(["ad_kernels.hip", "ad_gemm.hip", "ad_attention.hip", "ad_layer_fused.hip", "ad_sample.hip", "ad_host.cpp", "ad_sched.cpp"])
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in p.stdout.splitlines() if "packed-fp32-ops" not in l)
    if p.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if out.strip():
        print(out)
    os.replace(LIB + ".tmp", LIB)
    return LIB


def build_sched_test(force=True):
    if not force and not _stale(SCHED_LIB, _all_deps()):
        return SCHED_LIB
    cmd = ["g++", "-O2", "-std=c++17", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", SCHED_LIB + ".tmp"] + \
        _sources(["ad_sched.cpp", "ad_sched_testhook.cpp"])
    subprocess.run(cmd, check=True)
    os.replace(SCHED_LIB + ".tmp", SCHED_LIB)
    return SCHED_LIB


def build(force=True):
    return build_hip(force), build_sched_test(force)


if __name__ == "__main__":
    print(build(force="--if-stale" not in sys.argv))
