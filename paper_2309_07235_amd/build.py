"""Builds the HIP shared library in-tree: ``python -m paper_2309_07235_amd.build``.

The GEMM menu is compiled one translation unit per (element type, macro-tile),
generated from ``csrc/gemm_inst.hip.in``; objects are cached under ``_build/``
keyed by a hash of their inputs and compiled in parallel.
"""
from __future__ import annotations

import concurrent.futures
import hashlib
import os
import re
import subprocess
import sys
from pathlib import Path

HERE = Path(__file__).resolve().parent
CSRC = HERE / "csrc"
BUILD = HERE / "_build"
LIB = HERE / "libdla_mi355x.so"

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17", "-Wall", "-Wno-unused-function",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # no packed fp32 VALU ops
    "-mllvm", "-amdgpu-mfma-vgpr-form=1",                           # MFMA accumulators stay in VGPRs
]


def _tile_menu():
    text = (CSRC / "gemm_dispatch.hpp").read_text()
    body = text.split("#define DLA_TILE_MENU(X)")[1].split("\n\n")[0]
    return [tuple(int(v) for v in m.groups()) for m in re.finditer(r"X\((\d+), (\d+), (\d+), (\d+)\)", body)]


GEMM_HEADERS = ("dla_common.hpp", "gemm_kernel.hpp", "gemm_dispatch.hpp", "dla_codes.hpp")


def _headers_hash(gemm_only: bool = False) -> str:
    h = hashlib.sha256()
    headers = [CSRC / n for n in GEMM_HEADERS] if gemm_only else sorted(CSRC.glob("*.hpp"))
    for p in list(headers) + [HERE.parent / "include" / "dla.h"]:
        h.update(p.read_bytes())
    h.update(" ".join(FLAGS).encode())
    return h.hexdigest()


def _compile(src: Path, obj: Path, stamp: str, verbose: bool) -> str:
    tag = obj.with_suffix(".stamp")
    if obj.exists() and tag.exists() and tag.read_text() == stamp:
        return f"cached   {obj.name}"
    cmd = [HIPCC, *FLAGS, "-I", str(CSRC), "-c", str(src), "-o", str(obj)]
    res = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l and l.strip())
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src.name}:\n{err}")
    if verbose and err:
        print(err, file=sys.stderr)
    tag.write_text(stamp)
    return f"compiled {obj.name}"


def build(verbose: bool = False, jobs: int | None = None) -> Path:
    BUILD.mkdir(exist_ok=True)
    hh_all, hh_gemm = _headers_hash(False), _headers_hash(True)
    units = []
    template = (CSRC / "gemm_inst.hip.in").read_text()
    for tname, ctype in (("f64", "double"), ("f32", "float")):
        for tm, tn, wm, wn in _tile_menu():
            text = (template.replace("@T@", ctype).replace("@TM@", str(tm)).replace("@TN@", str(tn))
                    .replace("@WM@", str(wm)).replace("@WN@", str(wn)))
            src = BUILD / f"gemm_inst_{tname}_{tm}x{tn}_{wm}x{wn}.hip"
            if not src.exists() or src.read_text() != text:
                src.write_text(text)
            units.append(src)
    units += sorted(CSRC.glob("*.hip"))
    jobs = jobs or min(8, os.cpu_count() or 1)
    objs = []
    with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as ex:
        futs = []
        for src in units:
            obj = BUILD / (src.stem + ".o")
            hh = hh_gemm if src.name.startswith("gemm_") else hh_all
            stamp = hashlib.sha256((hh + src.read_text()).encode()).hexdigest()
            objs.append(obj)
            futs.append(ex.submit(_compile, src, obj, stamp, verbose))
        for f in futs:
            msg = f.result()
            if verbose:
                print(msg)
    tmp = LIB.with_suffix(f".so.tmp{os.getpid()}")
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", str(tmp), *map(str, objs)]
    subprocess.run(cmd, check=True)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
