"""Builds libf3m.so (the C-ABI HIP library) in-tree for gfx950 with hipcc."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJDIR = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libf3m.so")
RATES = os.path.join(HERE, "f3m_rates")
SOURCES = ["api.hip", "plan.hip", "kmvm.hip", "m2l.hip", "solve.hip", "pool.hip", "route.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         # packed FP32 instructions are not to be generated on the test machines
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # MFMA results go to ordinary VGPRs (gfx950 has a unified file): no v_accvgpr_read per value
         "-mllvm", "-amdgpu-mfma-vgpr-form"]


def _hipcc():
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def build_lib(verbose=False):
    os.makedirs(OBJDIR, exist_ok=True)
    hipcc = _hipcc()

    def compile_one(src):
        obj = os.path.join(OBJDIR, src.replace(".hip", ".o"))
        cmd = [hipcc, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        res = subprocess.run(cmd, capture_output=True, text=True)
        # the host pass warns that it does not know the packed-fp32 feature: harmless
        err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
        if res.returncode != 0:
            raise RuntimeError("hipcc failed for %s:\n%s" % (src, res.stderr))
        if err.strip():     # compiler warnings are always shown: they have pointed at real faults
            print(err, flush=True)
        return obj

    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n" + res.stderr)
    # the stand-alone rate probe (instruction and copy rates of the device, see csrc/rates.hip)
    res = subprocess.run([hipcc, *FLAGS, os.path.join(CSRC, "rates.hip"), "-o", RATES], capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed for rates.hip:\n" + res.stderr)
    return LIB


if __name__ == "__main__":
    print(build_lib(verbose="-v" in sys.argv))
