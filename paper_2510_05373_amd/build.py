"""Builds libkvlinc.so (the C-ABI library) and libkvlinc_probe.so (the benchmark's read-only probe kernel) in-tree with
hipcc for gfx950."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB_PATH = os.path.join(HERE, "libkvlinc.so")
PROBE_PATH = os.path.join(HERE, "libkvlinc_probe.so")

COMMON = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]
# per-file extras: the append path holds the bit-exact contracts, no contraction of a*b+c there
SOURCES = {
    "kvlinc_api.hip": [],
    "kvlinc_append.hip": ["-ffp-contract=off"],
    "kvlinc_decode.hip": [],
}
PROBE_SOURCE = "kvlinc_readprobe.hip"


def build(verbose=False):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    procs = []
    for src, extra in SOURCES.items():
        obj = os.path.join(CSRC, src.replace(".hip", ".o"))
        cmd = [hipcc] + COMMON + extra + ["-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    probe_cmd = [hipcc] + COMMON + ["-shared", os.path.join(CSRC, PROBE_SOURCE), "-o", PROBE_PATH]
    procs.append((PROBE_SOURCE, subprocess.Popen(probe_cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    for src, p in procs:
        out, _ = p.communicate()
        if p.returncode != 0:
            raise RuntimeError("hipcc failed on %s:\n%s" % (src, out))
        if verbose and out.strip():
            print(out)
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_PATH] + objs
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout)
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose=True))
