"""Compile the HIP sources under csrc/ into paper_1810_07354_amd/libscar.so for gfx950.

Each source file is compiled to an object of its own (in parallel; no device code calls
across files, so no relocatable device code is needed) and the objects are linked into the
shared library.  Objects live under _build/, which is not part of the repository."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libscar.so")
SOURCES = ["scar_api.hip", "scar_scores.hip", "scar_select.hip", "scar_rows.hip", "scar_var.hip",
           "scar_mixed.hip", "scar_store.hip", "scar_ceilings.hip"]
HEADERS = ["scar_device.hpp", "scar_host.hpp", os.path.join("..", "..", "include", "scar.h"),
           os.path.join("..", "..", "include", "scar_store.h"),
           os.path.join("..", "..", "include", "scar_ceilings.h")]

# Packed-FP32 instruction selection is switched off for all device code.
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-Wall", "-Wno-unused-function", "-pthread"]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(os.path.join(CSRC, f)) > t for f in SOURCES + HEADERS)


def _compile(hipcc, src, obj):
    subprocess.run([hipcc] + HIPCC_FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj], check=True)


def build(force: bool = True) -> str:
    """force: recompile every source; otherwise only the sources that changed since their
    object was made (all of them after a change to a header)."""
    if not force and not stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ_DIR, exist_ok=True)
    newest_header = max(os.path.getmtime(os.path.join(CSRC, h)) for h in HEADERS)
    jobs = []
    objs = []
    for src in SOURCES:
        obj = os.path.join(OBJ_DIR, src.replace(".hip", ".o"))
        objs.append(obj)
        fresh = (os.path.exists(obj) and os.path.getmtime(obj) >= os.path.getmtime(os.path.join(CSRC, src))
                 and os.path.getmtime(obj) >= newest_header)
        if force or not fresh:
            jobs.append((src, obj))
    with ThreadPoolExecutor(max_workers=min(8, max(1, len(jobs)))) as pool:
        for f in [pool.submit(_compile, hipcc, s, o) for s, o in jobs]:
            f.result()
    tmp = LIB + ".tmp.%d" % os.getpid()
    subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-pthread", "-o", tmp] + objs, check=True)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(force="--incremental" not in sys.argv))
    sys.exit(0)
