"""Build the gfx950 shared library ``libespresso_hip.so`` in-tree with hipcc.

``python -m paper_1705_07175_amd.build`` compiles every source under ``csrc/``
for ``--offload-arch=gfx950`` (hipcc cross-compiles without a GPU) and links
them next to this file, where the Python binding loads the library from.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(HERE, "_build")
LIB_PATH = os.path.join(HERE, "libespresso_hip.so")

# (source, extra flags).  host.cpp evaluates the batch-norm expression and must round after
# every operation, hence no fused multiply-add there.
SOURCES = (
    ("bgemm.hip", ()),
    ("bgemm_mfma.hip", ()),
    ("pack.hip", ()),
    ("conv.hip", ()),
    ("bconv_patch.hip", ()),
    ("float_layers.hip", ()),
    ("bitplane.hip", ()),
    ("probe.hip", ()),
    ("host.cpp", ("-ffp-contract=off",)),
)

COMMON = (
    "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-command-line-argument",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
)
# Device code: gfx950 only; packed-fp32 instruction selection is switched off.
DEVICE = ("--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops")


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


def _compile(job):
    src, extra = job
    obj = os.path.join(OBJ_DIR, os.path.splitext(src)[0] + ".o")
    cmd = [_hipcc(), *COMMON, *extra]
    if src.endswith(".hip"):
        cmd += list(DEVICE)
    cmd += ["-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # the host pass does not know the device-only target feature; that warning is noise
    out = "\n".join(l for l in res.stdout.splitlines()
                    if "packed-fp32-ops" not in l and l.strip())
    if res.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, res.stdout))
    return obj, out


def build(verbose: bool = False) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as pool:
        results = list(pool.map(_compile, SOURCES))
    if verbose:
        for _, out in results:
            if out:
                print(out)
    objs = [o for o, _ in results]
    tmp = LIB_PATH + ".tmp.%d" % os.getpid()
    cmd = [_hipcc(), "-shared", "-fPIC", "--offload-arch=gfx950", "-o", tmp, *objs]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n%s" % res.stdout)
    os.replace(tmp, LIB_PATH)
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
