"""Builds the HIP kernels into one shared library, in-tree, for gfx950 only.

    python -m paper_2505_11432_amd.build

hipcc cross-compiles without a GPU present.  The library is written next to this
file as libmoe_hip.so; the Python binding loads it with ctypes.
"""
from __future__ import annotations

import hashlib
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(HERE, "_build")
LIB_PATH = os.path.join(HERE, "libmoe_hip.so")
CEILINGS_SRC = os.path.join(CSRC, "ceilings", "ceilings.hip")       # measurement aids: a library of their own
CEILINGS_LIB_PATH = os.path.join(HERE, "libmoe_ceilings.so")
STAMP_PATH = LIB_PATH + ".sha256"      # hash of the sources the library was built from
INCLUDE = os.path.join(os.path.dirname(HERE), "include")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
COMMON_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed fp32 ALU forms have been unreliable on these boxes: keep the compiler from emitting them
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option", "-Wno-inline-asm",
]


def sources() -> list[str]:
    return sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hip"))


def source_hash() -> str:
    """SHA-256 over every file the library is compiled from (kernels, internal headers, the public header) and
    the compiler flags."""
    h = hashlib.sha256(" ".join(COMMON_FLAGS).encode())
    files = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith((".hip", ".h"))]
    files += [os.path.join(INCLUDE, f) for f in os.listdir(INCLUDE) if f.endswith(".h")]
    files.append(CEILINGS_SRC)
    for path in sorted(files):
        h.update(os.path.basename(path).encode())
        with open(path, "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()


def is_current() -> bool:
    """True when the library exists and was built from the sources as they are now."""
    if not (os.path.exists(LIB_PATH) and os.path.exists(CEILINGS_LIB_PATH) and os.path.exists(STAMP_PATH)):
        return False
    with open(STAMP_PATH) as fh:
        return fh.read().strip() == source_hash()


def ensure_built() -> str:
    """Build unless an up-to-date library is there: a library left over from older sources is rebuilt, never used."""
    if not is_current():
        build(verbose=False)
    return LIB_PATH


def _compile(src: str) -> str:
    obj = os.path.join(OBJ_DIR, os.path.basename(src)[:-4] + ".o")
    cmd = [HIPCC, *COMMON_FLAGS, "-c", src, "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    if os.path.exists(STAMP_PATH):
        os.remove(STAMP_PATH)           # no stamp while the library and the sources may disagree
    stamp = source_hash()
    srcs = sources()
    with ThreadPoolExecutor(max_workers=min(8, len(srcs) + 1)) as pool:
        ceil_obj = pool.submit(_compile, CEILINGS_SRC)
        objs = list(pool.map(_compile, srcs))
        ceil_obj = ceil_obj.result()
    res = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", CEILINGS_LIB_PATH, ceil_obj],
                         capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"link failed:\n{res.stderr}")
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_PATH, *objs]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"link failed:\n{res.stderr}")
    with open(STAMP_PATH, "w") as fh:
        fh.write(stamp + "\n")
    if verbose:
        print(f"built {LIB_PATH} from {len(srcs)} sources")
    return LIB_PATH


if __name__ == "__main__":
    build()
