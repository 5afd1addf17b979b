"""Build libmbconv.so (HIP, gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libmbconv.so")
SOURCES = ["mbconv_api.hip", "kernels_gemm.hip", "kernels_big.hip", "kernels_bf.hip", "kernels_x3.hip", "kernels_wave.hip", "kernels_pv16.hip", "kernels_dw.hip", "kernels_dw4.hip", "kernels_dw2.hip", "kernels_dwr.hip", "kernels_misc.hip"]
# sources without a block activation (Mish, layer normalisation, softmax): compiled once
SOURCES_ONCE = ["kernels_ops.hip"]
# packed fp32 VALU ops are disabled for the device pass (the host pass does not know the
# feature and says so; harmless)
FLAGS = ["--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


def build(force: bool = True, verbose: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    hipcc = _hipcc()
    headers = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    headers.append(os.path.join(HERE, "..", "include", "mbconv.h"))
    newest_hdr = max(os.path.getmtime(h) for h in headers)

    def compile_one(job) -> str:
        src, relu6 = job
        s = os.path.join(CSRC, src)
        o = os.path.join(OBJ, src.replace(".hip", "_r6.o" if relu6 else ".o"))
        if not force and os.path.exists(o) and os.path.getmtime(o) > max(os.path.getmtime(s), newest_hdr):
            return o
        # second pass: the same sources with ReLU6 as the block activation, in namespace mbk_r6
        extra = ["-DMBK_ACT_RELU6=1", "-Dmbk=mbk_r6"] if relu6 else []
        cmd = [hipcc, *FLAGS, *extra, "-c", s, "-o", o]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0 or verbose:
            sys.stderr.write(r.stdout + r.stderr)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}")
        return o

    jobs = [(src, relu6) for relu6 in (False, True) for src in SOURCES]
    jobs += [(src, False) for src in SOURCES_ONCE]
    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 4)) as ex:
        objs = list(ex.map(compile_one, jobs))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(r.stdout + r.stderr)
        raise RuntimeError("link failed")
    return LIB


if __name__ == "__main__":
    print(build(force="--incremental" not in sys.argv, verbose=True))
