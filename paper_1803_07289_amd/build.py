"""Build libflexconv.so (HIP, gfx950) in-tree with hipcc.

    python -m paper_1803_07289_amd.build [--force]

Objects go to _build/ (ignored by git), the shared library next to this file.
"""
import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(ROOT, "_build")
LIB = os.path.join(HERE, "libflexconv.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         # packed fp32 VALU ops are kept off on the test machines
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-munsafe-fp-atomics", "-Wall", "-Wno-unused-function", "-Wno-unknown-attributes"]


def shapes():
    out = []
    for line in open(os.path.join(CSRC, "flex_shapes.def")):
        m = re.match(r"\s*FLEX_SHAPE\(\s*(\d+)\s*,\s*(\d+)\s*,\s*(\d+)\s*,\s*(\d+)\s*,\s*(\d+)\s*,\s*(\d+)\s*\)", line)
        if m:
            out.append(tuple(int(x) for x in m.groups()))
    return out


def _jobs():
    jobs = []
    for name in ("flex_api", "flex_misc", "flex_pool", "flex_inedges", "flex_upsample", "flex_idiss", "flex_knn",
                 "flex_calibrate"):
        jobs.append((os.path.join(CSRC, name + ".hip"), os.path.join(OBJ, name + ".o"), []))
    for (di, do, w, t, occ, ws) in shapes():
        jobs.append((os.path.join(CSRC, "flex_tiled_inst.hip"),
                     os.path.join(OBJ, f"flex_tiled_{di}_{do}.o"),
                     [f"-DFLEX_DI={di}", f"-DFLEX_DO={do}", f"-DFLEX_W={w}", f"-DFLEX_T={t}", f"-DFLEX_OCC={occ}", f"-DFLEX_WS={ws}"]))
    return jobs


def _compile(job):
    src, obj, defs = job
    cmd = [HIPCC] + FLAGS + defs + ["-c", src, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l and l.strip())
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src} {defs}:\n{err}")
    return err


def build(force=True, jobs=8, verbose=False):
    os.makedirs(OBJ, exist_ok=True)
    todo = _jobs()
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        for msg in ex.map(_compile, todo):
            if verbose and msg:
                print(msg)
    objs = [j[1] for j in todo]
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
