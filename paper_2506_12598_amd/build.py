"""Builds libeclip.so (HIP kernels + C ABI) for gfx950 with hipcc: `python -m paper_2506_12598_amd.build`."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libeclip.so")
SOURCES = ["eclip.cpp", "alloc_solver.cpp", "k_gemm.hip", "k_wsk.hip", "k_mem.hip", "k_attn.hip", "k_gconv.hip"]


def pp_tile_ids():
    """Ids of the ping-pong tile shapes listed in gemm_tile.h; k_gemm_pp.hip is compiled once per id."""
    import re
    text = open(os.path.join(CSRC, "gemm_tile.h")).read()
    body = text[text.index("#define ECLIP_PP_TILES(X)"):]
    body = body[:body.index("\n\n")]
    return [int(v) for v in re.findall(r"X\((\d+),", body)]
FLAGS = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang",
         "-packed-fp32-ops", "-Wall", "-Wno-unused-function", "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _needs(obj: str, deps) -> bool:
    return not os.path.exists(obj) or any(os.path.getmtime(d) > os.path.getmtime(obj) for d in deps)


def build(force: bool = False, verbose: bool = False) -> str:
    bdir = os.path.join(HERE, "_build")
    os.makedirs(bdir, exist_ok=True)
    headers = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")] + [os.path.join(ROOT, "include", "eclip.h")]

    def compile_one(job):
        src, defs, tag = job
        path = os.path.join(CSRC, src)
        obj = os.path.join(bdir, src + tag + ".o")
        if force or _needs(obj, [path] + headers):
            cmd = ["hipcc", "-x", "hip", "-c", path, "-o", obj] + FLAGS + defs
            r = subprocess.run(cmd, capture_output=True, text=True)
            err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
            if r.returncode != 0:
                raise RuntimeError(f"hipcc failed on {src}:\n{err}")
            if verbose and err.strip():
                print(err, file=sys.stderr)
        return obj

    # the slowest translation units first, so that the pool stays full to the end
    jobs = [("k_gemm_pp.hip", [f"-DECLIP_PP_ID={i}"], f".{i}") for i in pp_tile_ids()] + [(src, [], "") for src in SOURCES]
    with ThreadPoolExecutor(max_workers=8) as ex:
        objs = list(ex.map(compile_one, jobs))
    if force or _needs(LIB, objs):
        r = subprocess.run(["hipcc", "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + objs, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("link failed:\n" + r.stderr)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv, verbose=True))
