"""Builds csrc/ into libtgemm.so for gfx950 with hipcc (in-tree, next to this file)."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
OBJ = os.path.join(_HERE, "_build")
LIB = os.path.join(_HERE, "libtgemm.so")

SOURCES = ["api.cpp", "plan.cpp", "engine.cpp", "mlp.hip", "gemm_f32.hip", "balance.hip", "gemm_bf16.hip", "gemm_bf16_dl.hip", "copy_kernel.hip"]

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950",
    # packed fp32 VALU forms are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument", "-Wno-unknown-attributes",
]


def _hipcc():
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.isabs(c) and os.path.exists(c) or not os.path.isabs(c)):
            return c
    raise RuntimeError("hipcc not found")


def _spilling_kernels(log):
    """Kernels whose resource remarks report private (scratch) memory: the GEMM kernels keep their
    accumulators in registers, and an accumulator array that the compiler moves to scratch (a loop it
    did not unroll, an index it could not resolve) still computes the right result, several times slower."""
    bad, name = [], None
    for line in log.splitlines():
        if "Function Name:" in line:
            name = line.split("Function Name:")[1].split("[")[0].strip()
        elif "ScratchSize [bytes/lane]:" in line:
            n = int(line.split("ScratchSize [bytes/lane]:")[1].split("[")[0])
            if n > 0:
                bad.append("%s: %d bytes per lane" % (name, n))
    return bad


def _compile(src):
    obj = os.path.join(OBJ, src + ".o")
    cmd = [_hipcc(), "-x", "hip"] + HIPCC_FLAGS + ["-Rpass-analysis=kernel-resource-usage",
                                                   "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    spills = _spilling_kernels(r.stdout)
    lines, skip = [], 0
    for l in r.stdout.splitlines():          # drop the resource remarks (each followed by a source excerpt)
        if "-Rpass-analysis=kernel-resource-usage" in l:
            skip = 2
            continue
        if skip and (l.lstrip().startswith(("|", "^")) or "|" in l[:12]):
            skip -= 1
            continue
        skip = 0
        lines.append(l)
    out = "\n".join(l for l in lines if "packed-fp32-ops" not in l and "warning generated" not in l
                    and "remark generated" not in l and "remarks generated" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, out))
    if spills:
        raise RuntimeError("%s: kernels use scratch memory:\n  %s" % (src, "\n  ".join(spills)))
    if out.strip():
        sys.stderr.write(out + "\n")
    return obj


def build(verbose=False):
    """Compiles every source (always) and links libtgemm.so.  Returns the library path."""
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES))
    tmp = LIB + ".tmp%d" % os.getpid()
    cmd = [_hipcc(), "-shared", "-fPIC", "--offload-arch=gfx950", "-o", tmp] + objs + ["-lpthread"]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout)
    os.replace(tmp, LIB)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
