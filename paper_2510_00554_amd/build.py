"""Build the gfx950 shared library ``libsentry_hip.so`` in-tree with hipcc."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsentry_hip.so")
SOURCES = ["sentry_host.hip", "sha256_merkle.hip", "blake2_lthash.hip", "blake2_lthash32.hip", "blake2_model.hip", "merkle_other.hip", "merkle_coalesce.hip", "sentry_stream.hip"]
# synthetic-input fill kernels for tests and bench.py: a library of its own, not part of the product
WORKLOADS_LIB = os.path.join(HERE, "libsentry_workloads.so")
WORKLOADS_SOURCE = "workloads_fill.hip"
# VALU issue-rate probe behind bench.py's roofline denominators: measurement plumbing, its own library too
PROBE_LIB = os.path.join(HERE, "libsentry_probe.so")
PROBE_SOURCE = "valu_probe.hip"
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]


def hipcc():
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.isabs(c) and os.path.exists(c) or not os.path.isabs(c)):
            return c
    return "hipcc"


def build(verbose=False):
    """Compile every HIP source for gfx950 and link the shared library.  Always compiles."""
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(CSRC, src.replace(".hip", ".o"))
        cmd = [hipcc()] + FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    failed = False
    for src, p in procs:
        out, _ = p.communicate()
        # hipcc's host pass does not know the gfx target feature and says so: harmless
        out = "\n".join(ln for ln in out.splitlines() if "packed-fp32-ops" not in ln)
        if p.returncode != 0:
            failed = True
            sys.stderr.write("hipcc failed on %s:\n%s\n" % (src, out))
        elif verbose and out.strip():
            print(out)
    if failed:
        raise RuntimeError("hipcc failed")
    tmp = LIB + ".tmp.%d" % os.getpid()
    cmd = [hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs
    subprocess.run(cmd, check=True)
    os.replace(tmp, LIB)
    tmp = WORKLOADS_LIB + ".tmp.%d" % os.getpid()
    cmd = [hipcc()] + FLAGS + ["-shared", os.path.join(CSRC, WORKLOADS_SOURCE), "-o", tmp]
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if p.returncode != 0:
        sys.stderr.write(p.stdout)
        raise RuntimeError("hipcc failed on " + WORKLOADS_SOURCE)
    os.replace(tmp, WORKLOADS_LIB)
    tmp = PROBE_LIB + ".tmp.%d" % os.getpid()
    cmd = [hipcc()] + FLAGS + ["-shared", os.path.join(CSRC, PROBE_SOURCE), "-o", tmp]
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if p.returncode != 0:
        sys.stderr.write(p.stdout)
        raise RuntimeError("hipcc failed on " + PROBE_SOURCE)
    os.replace(tmp, PROBE_LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
