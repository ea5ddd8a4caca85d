"""Builds the gfx950 generation library (csrc/*.hip -> librl_gen.so) with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "librl_gen.so")
SOURCES = ("elementwise.hip", "gemm_skinny.hip", "gemm_tiled.hip", "gemm_packed.hip", "attention_decode.hip", "attention_decode_gqa.hip", "attention_prefill.hip",
           "rl_gen.hip")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _headers_mtime() -> float:
    paths = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    inc = os.path.join(os.path.dirname(HERE), "include")
    paths += [os.path.join(inc, f) for f in os.listdir(inc)]
    return max(os.path.getmtime(p) for p in paths)


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    newest = max([_headers_mtime()] + [os.path.getmtime(os.path.join(CSRC, s)) for s in SOURCES])
    return os.path.getmtime(LIB) < newest


def build(force: bool = True, verbose: bool = False) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    hdr = _headers_mtime()

    def compile_one(src: str) -> str:
        s = os.path.join(CSRC, src)
        o = os.path.join(OBJ_DIR, src.replace(".hip", ".o"))
        if force or not os.path.exists(o) or os.path.getmtime(o) < max(os.path.getmtime(s), hdr):
            cmd = ["hipcc", *FLAGS, "-c", s, "-o", o]
            r = subprocess.run(cmd, capture_output=True, text=True)
            err = "\n".join(l for l in r.stderr.splitlines() if "is not a recognized feature" not in l)
            if r.returncode != 0:
                raise RuntimeError(f"hipcc failed for {src}:\n{err}")
            if verbose and err.strip():
                print(err)
        return o

    with ThreadPoolExecutor(max_workers=6) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    r = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    return LIB


def build_host_sanitize_check() -> str:
    """csrc/rl_gen.hip -- the host logic of the C ABI: validation, sizing, page planning, sequencing -- compiled with
    AddressSanitizer and UndefinedBehaviorSanitizer on the host side, plus csrc/host_sanitize_check.cpp, linked into one
    executable; the kernel launchers of the other sources come from the regular librl_gen.so (built first).  CPU only: the
    check launches nothing.  Takes a few seconds."""
    if not os.path.exists(LIB):
        build(force=False)
    out_dir = os.path.join(OBJ_DIR, "host_sanitize")
    os.makedirs(out_dir, exist_ok=True)
    inc = os.path.join(os.path.dirname(HERE), "include")
    san = ["-O1", "-g", "-std=c++17", "-fno-omit-frame-pointer", "-fno-sanitize-recover=all"]
    host_san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined"]
    rl = os.path.join(out_dir, "rl_gen.o")
    chk = os.path.join(out_dir, "host_sanitize_check.o")
    exe = os.path.join(out_dir, "host_sanitize_check")
    cmds = [
        ["hipcc", "--offload-arch=gfx950", *san, *host_san, "-fPIC", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-c", os.path.join(CSRC, "rl_gen.hip"), "-o", rl],
        # plain C++ (hipcc would treat it as HIP): the host compiler that hipcc drives
        ["/opt/rocm/lib/llvm/bin/clang++", *san, "-fsanitize=address", "-fsanitize=undefined", "-I", inc, "-c",
         os.path.join(CSRC, "host_sanitize_check.cpp"), "-o", chk],
        ["hipcc", "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-Wno-option-ignored", "-o", exe, rl, chk,
         LIB, "-Wl,-rpath," + HERE],
    ]
    for cmd in cmds:
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("failed: " + " ".join(cmd) + "\n" + r.stderr)
    return exe


if __name__ == "__main__":
    import sys
    print(build(force="--incremental" not in sys.argv, verbose=True))
