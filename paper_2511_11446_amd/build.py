"""Build the HIP library for gfx950, in-tree: python -m paper_2511_11446_amd.build"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJDIR = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libdiffpro_qlinear.so")
SOURCES = ["daq.hip", "daq_robust.hip", "daq_ln.hip", "qgemm.hip", "qgemm_w4.hip", "offline_host.hip", "api.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17",
    "-ffp-contract=off",                            # every fused multiply-add in the kernels is written out
    "-fhip-fp32-correctly-rounded-divide-sqrt",      # DAQ needs the IEEE quotient
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def _compile(src):
    obj = os.path.join(OBJDIR, src.replace(".hip", ".o"))
    cmd = [HIPCC, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops' is not a recognized feature" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, out))
    if out.strip():
        print(out, file=sys.stderr)
    return obj


def build(verbose=True):
    os.makedirs(OBJDIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        objs = list(ex.map(_compile, SOURCES))
    tmp = LIB + ".tmp%d" % os.getpid()
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", tmp,
                           "-Wno-unused-command-line-argument"])
    os.replace(tmp, LIB)
    if verbose:
        print("built", LIB)
    return LIB


# bench.py's measurement aid (a register-resident MFMA loop): a shared object of its own beside bench.py, not in the library
PROBE_SRC = os.path.join(os.path.dirname(HERE), "bench_mfma_probe.hip")
PROBE_LIB = os.path.join(os.path.dirname(HERE), "libbench_mfma_probe.so")


def build_bench_probe(verbose=True):
    tmp = PROBE_LIB + ".tmp%d" % os.getpid()
    r = subprocess.run([HIPCC, *FLAGS, "-shared", PROBE_SRC, "-o", tmp], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (PROBE_SRC, r.stdout))
    os.replace(tmp, PROBE_LIB)
    if verbose:
        print("built", PROBE_LIB)
    return PROBE_LIB


if __name__ == "__main__":
    build()
    build_bench_probe()
