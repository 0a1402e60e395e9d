"""Build libconserve_kv.so for gfx950 with hipcc (cross-compiles without a GPU)."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.path.join(HERE, "libconserve_kv.so")
SOURCES = ["cs_api.hip", "cs_copy_kernels.hip", "cs_decode.hip", "cs_prefill.hip", "cs_mixed.hip", "cs_page_map.hip", "cs_static_scratch.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-I", INCLUDE, "-I", CSRC,
    # packed fp32 arithmetic stays off: the compiler must not form v_pk_*_f32
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def _compile(src, extra):
    obj = os.path.join(CSRC, src.replace(".hip", ".o"))
    subprocess.check_call(["hipcc", *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj])
    return obj


def build(extra_flags=()) -> str:
    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(lambda s: _compile(s, list(extra_flags)), SOURCES))
    tmp = LIB + ".tmp.%d" % os.getpid()
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", tmp])
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(sys.argv[1:]))
