"""Builds libsev.so (HIP, gfx950 only) in-tree with hipcc."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsev.so")
SOURCES = ["sev_api.hip", "kernels_common.hip", "kernels_f32.hip", "kernels_bf16.hip", "sev_sched.cpp"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang",
         "-packed-fp32-ops", "-Wno-unused-command-line-argument", "-Wno-unused-value", "-Wno-unused-result",
         # the first 16 dwords of a kernel's scalar arguments arrive in registers at wave launch (no scalar load of
         # the argument block on the critical path of the prologue); kernels list what they need first in front
         "-mllvm", "-amdgpu-kernarg-preload-count=16"]


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    procs = []
    bdir = os.path.join(HERE, "_build")
    os.makedirs(bdir, exist_ok=True)
    for s in SOURCES:
        o = os.path.join(bdir, os.path.splitext(s)[0] + ".o")
        objs.append(o)
        cmd = [hipcc, *FLAGS, "-c", os.path.join(CSRC, s), "-o", o]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((s, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    failed = False
    for s, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            failed = True
            sys.stderr.write(f"--- {s} failed ---\n{out}\n")
        elif verbose and out.strip():
            print(out)
    if failed:
        raise RuntimeError("hipcc failed")
    subprocess.check_call([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs])
    return LIB


def build_host_sanitized(out_dir: str) -> str:
    """Builds tests/host_sanitize/driver.cpp together with every source of the library and synth/rng.c, with
    AddressSanitizer and UndefinedBehaviorSanitizer on the HOST code only (device code is compiled as usual: the GPU
    sanitizers are not used), into out_dir/host_sanitize.  The program needs no GPU."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    clang = os.path.join(os.path.dirname(os.path.realpath(hipcc)), "..", "llvm", "bin", "clang")
    if not os.path.exists(clang):
        clang = "/opt/rocm/llvm/bin/clang"
    root = os.path.dirname(HERE)
    os.makedirs(out_dir, exist_ok=True)
    san = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined", "-g"]
    host_only = [x for f in san for x in ("-Xarch_host", f)]
    jobs = []
    for s in SOURCES:
        o = os.path.join(out_dir, os.path.splitext(s)[0] + ".o")
        if s.endswith(".hip"):
            cmd = [hipcc, "--offload-arch=gfx950", "-O1", "-std=c++17", *host_only, "-Xclang", "-target-feature", "-Xclang",
                   "-packed-fp32-ops", "-Wno-unused-command-line-argument", "-Wno-unused-value", "-Wno-unused-result",
                   "-Wno-pass-failed", "-c", os.path.join(CSRC, s), "-o", o]
        else:
            cmd = [clang + "++", "-std=c++17", "-O1", *san, "-c", os.path.join(CSRC, s), "-o", o]
        jobs.append((o, cmd))
    jobs.append((os.path.join(out_dir, "rng.o"), [clang, "-O1", *san, "-c", os.path.join(root, "synth", "rng.c"), "-o",
                                                  os.path.join(out_dir, "rng.o")]))
    jobs.append((os.path.join(out_dir, "driver.o"), [clang + "++", "-std=c++17", "-O1", *san, "-c",
                                                     os.path.join(root, "tests", "host_sanitize", "driver.cpp"), "-o",
                                                     os.path.join(out_dir, "driver.o")]))
    procs = [(o, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)) for o, cmd in jobs]
    for o, p in procs:
        out, _ = p.communicate()
        if p.returncode != 0:
            raise RuntimeError(f"building {o} failed:\n{out}")
    exe = os.path.join(out_dir, "host_sanitize")
    subprocess.check_call([hipcc, "-fsanitize=address", "-fsanitize=undefined", *[o for o, _ in jobs], "-o", exe, "-lm"])
    return exe


if __name__ == "__main__":
    print(build(verbose=True))
