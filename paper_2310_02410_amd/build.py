"""Builds libmoqe.so (the C-ABI HIP library) in-tree for gfx950 with hipcc."""

from __future__ import annotations

import os
import shutil
import subprocess
import tempfile
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libmoqe.so")
SOURCES = ("moqe_api.hip", "moqe_quantize.hip", "moqe_route.hip", "moqe_ffn_decode.hip", "moqe_ffn_decode_small.hip",
           "moqe_ffn_prefill.hip", "moqe_ffn_resident.hip", "moqe_stream_read.hip")


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found; the MoQE library needs ROCm to build")
    return exe


def build_library(verbose: bool = False, extra=(), out: str = LIB) -> str:
    """Compile every HIP source (in parallel, one object each) and link them into
    paper_2310_02410_amd/libmoqe.so; always recompiles."""
    flags = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             # keep the four words of an unpacked MFMA fragment as scalar ops: the SLP vectorizer
             # would turn (a & mask) | magic into vector ops that no longer select v_and_or_b32
             "-fno-slp-vectorize",
             "-Wno-unused-command-line-argument",
             "-I", os.path.join(os.path.dirname(PKG), "include"), *extra]
    objdir = tempfile.mkdtemp(prefix="moqe_build_")
    try:
        def compile_one(src):
            obj = os.path.join(objdir, src + ".o")
            cmd = [hipcc(), *flags, "-c", os.path.join(CSRC, src), "-o", obj]
            if verbose:
                print(" ".join(cmd), flush=True)
            res = subprocess.run(cmd, capture_output=True, text=True)
            if res.returncode != 0:
                raise RuntimeError(f"hipcc failed on {src}:\n" + res.stdout + res.stderr)
            return obj

        with ThreadPoolExecutor(max_workers=min(len(SOURCES), os.cpu_count() or 1)) as pool:
            objs = list(pool.map(compile_one, SOURCES))
        cmd = [hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", out + ".tmp"]
        if verbose:
            print(" ".join(cmd), flush=True)
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError("link failed:\n" + res.stdout + res.stderr)
        os.replace(out + ".tmp", out)
    finally:
        shutil.rmtree(objdir, ignore_errors=True)
    return out


if __name__ == "__main__":
    print(build_library(verbose=True))
