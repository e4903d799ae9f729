"""Build libicq.so (the C-ABI HIP library) for gfx950 with hipcc, in-tree.

    python -m paper_1912_08756_amd.build

Objects go to _build/ (ignored); the shared library lands next to this file so
that it travels with the source tree.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OUT = os.path.join(HERE, "libicq.so")
BUILD_DIR = os.path.join(ROOT, "_build")
SOURCES = ["icq_index.hip", "icq_lut.hip", "icq_scan.hip", "icq_scan16.hip", "icq_group.hip", "icq_group2.hip", "icq_refine.hip", "icq_search.hip", "icq_running.hip", "icq_policy.hip", "icq_encode.hip", "icq_probe.hip"]
FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-fvisibility=hidden",
    "-Wall", "-Wno-unused-command-line-argument",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
]


def _compile(src):
    obj = os.path.join(BUILD_DIR, os.path.splitext(src)[0] + ".o")
    cmd = ["hipcc"] + FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines()
                    if "packed-fp32-ops" not in l or "not a recognized feature" not in l)
    return src, obj, r.returncode, out


def build(verbose=True):
    os.makedirs(BUILD_DIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        results = list(ex.map(_compile, SOURCES))
    objs = []
    for src, obj, rc, out in results:
        if out.strip() and verbose:
            print("[%s]\n%s" % (src, out))
        if rc != 0:
            raise RuntimeError("hipcc failed on %s" % src)
        objs.append(obj)
    tmp = OUT + ".tmp.%d" % os.getpid()
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs)
    os.replace(tmp, OUT)
    return OUT


if __name__ == "__main__":
    print(build())
    sys.exit(0)
