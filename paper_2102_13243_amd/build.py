"""Builds libs4tf.so (HIP kernels + C ABI) for gfx950, in tree."""
import concurrent.futures
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libs4tf.so")
SOURCES = ["igemm.hip", "igemm_dma.hip", "patchconv.hip", "dwconv.hip", "bn.hip", "pool.hip", "head.hip", "api.hip", "step.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wno-unused-function"]


def _compile(src):
    out = os.path.join(OBJ, src.replace(".hip", ".o"))
    cmd = ["hipcc", "-c", os.path.join(CSRC, src), "-o", out] + FLAGS
    res = subprocess.run(cmd, capture_output=True, text=True)
    text = "\n".join(l for l in (res.stdout + res.stderr).splitlines()
                     if "not a recognized feature for this target" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, text))
    return out, text


def build(verbose=False):
    os.makedirs(OBJ, exist_ok=True)
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        results = list(ex.map(_compile, SOURCES))
    if verbose:
        for _, text in results:
            if text.strip():
                print(text)
    objs = [o for o, _ in results]
    subprocess.check_call(["hipcc", "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + objs)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
