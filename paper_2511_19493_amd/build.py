"""Builds librfx.so (HIP, gfx950) in-tree with hipcc.

    python -m paper_2511_19493_amd.build [--force]

Objects go to paper_2511_19493_amd/_build/, the library to paper_2511_19493_amd/lib/librfx.so.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor
from pathlib import Path

PKG = Path(__file__).resolve().parent
ROOT = PKG.parent
CSRC = PKG / "csrc"
OBJ = PKG / "_build"
LIB = PKG / "lib" / "librfx.so"

HIPCC = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
    # packed-FP32 instruction forms are switched off for every device compilation
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    f"-I{ROOT / 'include'}", f"-I{CSRC}",
]


def _stale(target: Path, deps) -> bool:
    if not target.exists():
        return True
    t = target.stat().st_mtime
    return any(d.stat().st_mtime > t for d in deps)


# sources that are compiled several times, once per set of kernel instantiations: (object stem, extra flags)
VARIANTS = {
    "prox_dense.hip": [(f"prox_dense_mode{m}", [f"-DRFX_TILE_MODE={m}"]) for m in range(5)],
}


def build(force: bool = False, verbose: bool = True) -> Path:
    srcs = []
    for src in sorted(CSRC.glob("*.hip")):
        for stem, extra in VARIANTS.get(src.name, [(src.stem, [])]):
            srcs.append((src, stem, extra))
    # the longest compilations first
    srcs.sort(key=lambda t: (t[0].name not in VARIANTS and t[0].name != "grow.hip", t[1]))
    hdrs = sorted(CSRC.glob("*.h")) + sorted((ROOT / "include").glob("*.h"))
    OBJ.mkdir(exist_ok=True)
    LIB.parent.mkdir(exist_ok=True)

    def compile_one(job):
        src, stem, extra = job
        obj = OBJ / (stem + ".o")
        if force or _stale(obj, [src, *hdrs]):
            cmd = [HIPCC, *FLAGS, *extra, "-c", str(src), "-o", str(obj)]
            if verbose:
                print("[build]", " ".join(cmd), flush=True)
            r = subprocess.run(cmd, capture_output=True, text=True)
            msgs = "\n".join(l for l in (r.stdout + r.stderr).splitlines()
                             if "packed-fp32-ops" not in l and "argument unused" not in l)
            if r.returncode != 0:
                raise RuntimeError(f"hipcc failed on {src.name}:\n{msgs}")
            if verbose and msgs.strip():
                print(msgs, flush=True)
        return obj

    jobs = min(len(srcs), int(os.environ.get("MAX_JOBS", "8")), 16)
    with ThreadPoolExecutor(max_workers=max(1, jobs)) as ex:
        objs = list(ex.map(compile_one, srcs))
    for old in OBJ.glob("*.o"):      # objects of sources or variants that no longer exist
        if old not in objs:
            old.unlink()
    if force or _stale(LIB, objs):
        cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *map(str, objs), "-o", str(LIB)]
        if verbose:
            print("[build]", " ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
