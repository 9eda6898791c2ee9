"""Builds libavq.so (HIP, gfx950 only) in-tree with hipcc.

`python -m paper_1908_10396_amd.build` compiles every translation unit under
csrc/ and links them into paper_1908_10396_amd/libavq.so. hipcc cross-compiles
for gfx950 without a GPU present.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libavq.so")
UNITS = ["api", "lut", "scan", "scan_mfma", "refine", "select", "ivf", "layout", "train"]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17",
    "-ffp-contract=off",                      # the fp32 query path has a defined operation order
    "-fhip-fp32-correctly-rounded-divide-sqrt",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def _hipcc():
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.sep not in c or os.path.exists(c)):
            return c
    raise RuntimeError("hipcc not found")


def _newer(target, sources):
    if not os.path.exists(target):
        return False
    t = os.path.getmtime(target)
    return all(os.path.getmtime(s) <= t for s in sources)


def build(force=True, verbose=False, jobs=8):
    os.makedirs(OBJ, exist_ok=True)
    headers = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    headers.append(os.path.join(os.path.dirname(HERE), "include", "avq.h"))
    hipcc = _hipcc()

    def compile_one(u):
        src = os.path.join(CSRC, u + ".hip")
        obj = os.path.join(OBJ, u + ".o")
        if not force and _newer(obj, [src] + headers):
            return obj
        # -save-temps=obj leaves the device assembly beside the object: it is checked below, then the extras go
        cmd = [hipcc] + FLAGS + ["-save-temps=obj", "-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed for %s:\n%s\n%s" % (u, r.stdout, r.stderr))
        if verbose and r.stderr.strip():
            print(r.stderr, file=sys.stderr)
        _check_device_code(u)
        return obj

    def _check_device_code(u):
        # No 96-bit LDS access may be left in a kernel: a value of three adjacent words that one thread
        # published for its workgroup through such a store and load came out wrong now and then on MI355X
        # (the selection in wg_select.h; it publishes one 64-bit word since). The compiler forms these
        # accesses by itself from neighbouring 32-bit ones, so the check is on its output.
        asm = os.path.join(OBJ, u + "-hip-amdgcn-amd-amdhsa-gfx950.s")
        bad, kernel = [], "?"
        if os.path.exists(asm):
            with open(asm) as f:
                for line in f:
                    if line.startswith("_Z") and ":" in line:
                        kernel = line.split(":")[0]
                    elif "ds_read_b96" in line or "ds_write_b96" in line:
                        bad.append(kernel)
        for f in os.listdir(OBJ):
            if f.startswith(u + "-hip-") or f.startswith(u + "-host-") or f.startswith(u + ".hip-"):
                os.remove(os.path.join(OBJ, f))
        if bad:
            raise RuntimeError("%s.hip: 96-bit LDS accesses in %s" % (u, ", ".join(sorted(set(bad)))))

    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(compile_one, UNITS))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n%s\n%s" % (r.stdout, r.stderr))
    return LIB


if __name__ == "__main__":
    print(build(force="--incremental" not in sys.argv, verbose=True))
