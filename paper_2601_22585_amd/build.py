"""Builds libhcl.so for gfx950 with hipcc (in-tree, next to this file)."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libhcl.so")
SOURCES = ["hcl_api.cpp", "reduce_copy.hip", "ring_fused.hip", "static_scratch.hip"]   # ring_fused.hip is compiled once per wire type and part
HEADERS = ["reduce_copy.h", "ring_sched.h", "wire.h", "internal.h"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-fno-gpu-flush-denormals-to-zero", "-ffp-contract=off",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option",
]


def stale():
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in SOURCES + HEADERS] + [os.path.join(ROOT, "include", "hcl.h")]
    return any(os.path.getmtime(d) > t for d in deps)


def build_lib(force=True, verbose=False):
    """Compile the library.  force=False rebuilds only when a source is newer."""
    if not force and not stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    # translation units: the API, the step kernels, and the fused kernels once per
    # (wire type, part) -- compiled side by side, then one link
    units = [("hcl_api.cpp", "hcl_api", []), ("reduce_copy.hip", "reduce_copy", []),
             ("static_scratch.hip", "static_scratch", [])]
    for dt in range(7):
        for part in range(2):
            units.append(("ring_fused.hip", f"ring_fused_dt{dt}_p{part}", [f"-DHCL_FUSED_DT={dt}", f"-DHCL_FUSED_PART={part}"]))
    objs, cmds = [], []
    for src, name, defs in units:
        obj = os.path.join(objdir, name + ".o")
        cmds.append([hipcc, *HIPCC_FLAGS, *defs, "-I", os.path.join(ROOT, "include"), "-I", CSRC,
                     "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj])
        objs.append(obj)
    jobs = max(1, min(len(cmds), int(os.environ.get("MAX_JOBS", os.cpu_count() or 1))))
    running, pending = [], list(cmds)
    while pending or running:
        while pending and len(running) < jobs:
            cmd = pending.pop(0)
            if verbose:
                print(" ".join(cmd), flush=True)
            running.append((cmd, subprocess.Popen(cmd)))
        cmd, p = running.pop(0)
        if p.wait() != 0:
            for _, q in running:
                q.kill()
            raise subprocess.CalledProcessError(p.returncode, cmd)
    link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB]
    if verbose:
        print(" ".join(link), flush=True)
    subprocess.check_call(link)
    return LIB


EXAMPLES = ["allreduce_latency", "allreduce_from_file", "allreduce_bandwidth"]   # plain C against the library
PROBES = ["stream_ceilings"]   # stand-alone HIP programs that use no part of the library


def build_examples(verbose=False):
    """Compile the plain-C examples against the built library (they link libhcl.so by path)
    and the stand-alone HIP probes.  Returns the executables' paths."""
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    exes, cmds = [], []
    for name in EXAMPLES:
        src = os.path.join(HERE, "examples", name + ".c")
        exe = os.path.join(HERE, "examples", name)
        cmds.append(["gcc", "-O2", "-std=gnu11", "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(rocm, "include"),
                     "-I", os.path.join(ROOT, "include"), src, "-L", HERE, "-lhcl", "-L", os.path.join(rocm, "lib"), "-lamdhip64",
                     "-Wl,-rpath,$ORIGIN/..", "-Wl,-rpath," + os.path.join(rocm, "lib"), "-o", exe])
        exes.append(exe)
    for name in PROBES:
        exe = os.path.join(HERE, "examples", name)
        cmds.append([hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                     "-Wno-unknown-warning-option", os.path.join(HERE, "examples", name + ".hip"), "-o", exe])
        exes.append(exe)
    for cmd in cmds:
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.check_call(cmd)
    return exes


if __name__ == "__main__":
    build_lib(force=True, verbose=True)
    print(LIB)
    print("\n".join(build_examples(verbose=True)))
