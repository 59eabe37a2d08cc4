"""Compiles the HIP library for gfx950 in-tree:  python -m paper_2410_21120_amd.build"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OUT = os.path.join(HERE, "libfusedinf.so")
SOURCES = ["fi_plan.cpp", "fi_api.cpp", "fi_sched.cpp", "fi_server.cpp", "fi_kernels.hip", "fi_chain.hip", "fi_stem.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def sources():
    return [os.path.join(CSRC, s) for s in SOURCES]


def stale() -> bool:
    if not os.path.exists(OUT):
        return True
    t = os.path.getmtime(OUT)
    deps = sources() + [os.path.join(CSRC, "fi_internal.h"), os.path.join(CSRC, "fi_device.h"), os.path.join(HERE, "..", "include", "fusedinf.h")]
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = True) -> str:
    if not force and not stale():
        return OUT
    cmd = [HIPCC, *FLAGS, "-x", "hip", *sources(), "-o", OUT]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if out.strip():
        print(out)
    return OUT


if __name__ == "__main__":
    print("built", build())
