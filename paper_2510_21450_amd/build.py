"""Builds libpararnn.so (gfx950) in-tree with hipcc.

Each .hip file is compiled to an object on its own (in parallel) and linked
into paper_2510_21450_amd/libpararnn.so.  No GPU is needed to build.

`python -m paper_2510_21450_amd.build` builds the library and the example
cells under user_cells/; `--cell my_cell.hip [-o libmy_cell.so]` builds a
library for a cell written against include/pararnn_cell.h and links it
against libpararnn.so.
"""
from __future__ import annotations

import concurrent.futures as cf
import glob
import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libpararnn.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
INCLUDE = os.path.join(os.path.dirname(PKG), "include")      # public headers: pararnn.h, pararnn_cell.h, pararnn/*.h
FLAGS = ["--offload-arch=gfx950", f"-I{INCLUDE}", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
         # packed fp32 VALU forms are kept off for the test machines
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-inline-asm", "-Wno-unused-but-set-variable", "-Wno-unknown-warning-option",
         "-Wno-sometimes-uninitialized", "-Wno-uninitialized"]


USER_CELLS = os.path.join(PKG, "user_cells")


def _compile(src: str, extra) -> str:
    obj = os.path.join(OBJ, os.path.basename(src) + ".o")
    cmd = [HIPCC, *FLAGS, *extra, "-c", src, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{r.stderr}")
    noise = "packed-fp32-ops"
    warn = "\n".join(l for l in r.stderr.splitlines() if noise not in l and l.strip())
    if warn:
        sys.stderr.write(warn + "\n")
    return obj


def build(jobs: int | None = None, extra_flags=(), verbose: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    srcs = sorted(glob.glob(os.path.join(CSRC, "*.hip")))
    jobs = jobs or min(8, os.cpu_count() or 1)
    with cf.ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda s: _compile(s, list(extra_flags)), srcs))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-rdc", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    if verbose:
        print("built", LIB)
    return LIB


def build_cell(src: str, out: str | None = None, extra_flags=(), verbose: bool = False, obj: str | None = None) -> str:
    """Compile one .hip file that defines a cell (PARARNN_DEFINE_CELL) into a shared
    library next to libpararnn.so (or at `out`), linked against libpararnn.so.
    `obj`: an object file already compiled from `src` (only the link is done)."""
    if not os.path.exists(LIB):
        raise RuntimeError(f"{LIB} is missing: build the library first")
    os.makedirs(OBJ, exist_ok=True)
    stem = os.path.splitext(os.path.basename(src))[0]
    out = out or os.path.join(PKG, f"libpararnn_{stem}.so")
    obj = obj or _compile(src, list(extra_flags))
    rpath = "$ORIGIN" if os.path.dirname(os.path.abspath(out)) == PKG else PKG
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-rdc", "-o", out, obj,
           f"-L{PKG}", "-lpararnn", f"-Wl,-rpath,{rpath}"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    if verbose:
        print("built", out)
    return out


def build_examples(jobs: int | None = None, verbose: bool = False):
    """The example cells under user_cells/ (libpararnn_<name>.so beside the library)."""
    srcs = sorted(glob.glob(os.path.join(USER_CELLS, "*.hip")))
    with cf.ThreadPoolExecutor(max_workers=jobs or min(8, os.cpu_count() or 1)) as ex:
        return list(ex.map(lambda s: build_cell(s, verbose=verbose), srcs))


def build_all(jobs: int | None = None, verbose: bool = False):
    """The library and the example cells; the cells' objects compile alongside the library's (they
    only need the library at link time)."""
    os.makedirs(OBJ, exist_ok=True)
    cells = sorted(glob.glob(os.path.join(USER_CELLS, "*.hip")))
    with cf.ThreadPoolExecutor(max_workers=jobs or min(8, os.cpu_count() or 1)) as ex:
        # the slowest translation units first
        cell_objs = [ex.submit(_compile, s, []) for s in reversed(cells)]
        lib = ex.submit(build, jobs, (), verbose)
        lib.result()
        objs = [f.result() for f in cell_objs][::-1]
    return [build_cell(s, verbose=verbose, obj=o) for s, o in zip(cells, objs)]


if __name__ == "__main__":
    import argparse
    ap = argparse.ArgumentParser(description=__doc__)
    ap.add_argument("--cell", help="build only this user-cell source against the existing library")
    ap.add_argument("-o", "--out", help="output path of the user-cell library")
    args = ap.parse_args()
    if args.cell:
        build_cell(args.cell, args.out, verbose=True)
    else:
        build_all(verbose=True)
