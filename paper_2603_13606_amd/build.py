"""Builds libep_mi355x.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libep_mi355x.so")
SOURCES = ["ep_api.hip", "ep_layout.hip", "ep_dispatch.hip", "ep_dedup.hip", "ep_combine.hip", "ep_staged.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# packed-fp32 instructions are switched off on purpose: some of their forms have
# produced wrong results on the target machines.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-command-line-argument",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


HEADERS = [os.path.join(CSRC, "ep_internal.h"), os.path.join(CSRC, "ep_fp8.h"), os.path.join(ROOT, "include", "ep.h")]
_ID_MARK = b"EP_BUILD_ID="


def source_id() -> str:
    """16 hex digits naming the sources and flags the library is built from."""
    import hashlib
    h = hashlib.sha256()
    for path in [os.path.join(CSRC, s) for s in SOURCES] + HEADERS:
        h.update(os.path.basename(path).encode() + b"\0")
        with open(path, "rb") as f:
            h.update(f.read())
    h.update(" ".join(FLAGS[:-4]).encode())  # the include paths differ from tree to tree
    return h.hexdigest()[:16]


def built_id(lib: str = LIB):
    """The source id a built library carries (read from the file, which is not loaded), or None."""
    try:
        with open(lib, "rb") as f:
            data = f.read()
    except OSError:
        return None
    at = data.find(_ID_MARK)
    if at < 0:
        return None
    return data[at + len(_ID_MARK): at + len(_ID_MARK) + 16].decode("ascii", "replace")


def is_current() -> bool:
    """True when the library in the tree was built from the sources in the tree."""
    return built_id() == source_id()


def _compile(src: str) -> str:
    obj = os.path.join(CSRC, src.replace(".hip", ".o"))
    cmd = [HIPCC, *FLAGS, f'-DEP_BUILD_ID_STRING="{source_id()}"', "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{r.stdout}\n{r.stderr}")
    warn = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l and l.strip())
    if warn:
        sys.stderr.write(warn + "\n")
    return obj


def build(verbose: bool = False) -> str:
    """Compile every source and link the shared library; always recompiles."""
    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")
    if verbose:
        print(f"built {LIB}")
    return LIB


if __name__ == "__main__":
    build(verbose=True)
