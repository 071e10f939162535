"""Builds the HIP kernels and the C-ABI library (libchipmunk_hip.so) for gfx950, in-tree, and beside it the
device-ceiling probes that bench.py --ceilings times (libchipmunk_ceilings.so)."""
import glob
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libchipmunk_hip.so")
PROBE_SRC = os.path.join(HERE, "probe", "ceilings.hip")
PROBE_LIB = os.path.join(HERE, "libchipmunk_ceilings.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-fno-honor-nans",
    # hipcc -O3 must not form packed-fp32 instructions on this target
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def is_stale():
    if not os.path.exists(LIB):
        return True
    deps = sources() + glob.glob(os.path.join(CSRC, "*.h")) + [os.path.join(HERE, "..", "include", "chipmunk.h")]
    return any(os.path.getmtime(d) > os.path.getmtime(LIB) for d in deps)


def build(verbose=False):
    """Compile every .hip source into one shared library.  Always recompiles."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    procs = []
    for src in sources():
        obj = src[:-4] + ".o"
        cmd = [hipcc] + [f for f in HIPCC_FLAGS if f != "-shared"] + ["-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    failed = False
    for src, pr in procs:
        out, _ = pr.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if pr.returncode != 0:
            failed = True
            sys.stderr.write(f"hipcc failed on {src}:\n{out}\n")
        elif verbose and out.strip():
            print(out)
    if failed:
        raise RuntimeError("hipcc failed")
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    subprocess.run(cmd, check=True)
    for o in objs:
        os.remove(o)
    probe = subprocess.run([hipcc] + HIPCC_FLAGS + [PROBE_SRC, "-o", PROBE_LIB], stdout=subprocess.PIPE,
                           stderr=subprocess.STDOUT, text=True)
    if probe.returncode != 0:
        sys.stderr.write(probe.stdout)
        raise RuntimeError("hipcc failed on the ceiling probes")
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
