"""Build libcopris.so (gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libcopris.so")
OBJ_DIR = os.path.join(PKG_DIR, "_build")
SOURCES = ["copris_api.hip", "decode_attn.hip", "prefill_attn.hip", "lmhead.hip", "is_ratio.hip",
           "rollout_manager.cpp", "rollout_device.hip"]
# the host pass warns that it does not know the packed-fp32 feature: harmless
NOISE = ("is not a recognized feature", "1 warning generated", "warnings generated")


def hipcc_path() -> str:
    for cand in (os.environ.get("HIPCC"), shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


def compile_flags() -> list:
    return ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
            # packed-FP32 arithmetic is switched off for all device code
            "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
            "-Wno-unused-command-line-argument",
            "-I", os.path.join(os.path.dirname(PKG_DIR), "include")]


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stderr)
    err = "\n".join(l for l in res.stderr.splitlines() if not any(n in l for n in NOISE))
    if verbose and err.strip():
        print(err, file=sys.stderr)


def build(verbose: bool = False, lib_path: str = LIB_PATH, extra_flags=()) -> str:
    """Compile every HIP source for gfx950 (one hipcc process per file, side by side) and
    link the shared library."""
    hipcc = hipcc_path()
    os.makedirs(OBJ_DIR, exist_ok=True)
    tag = os.path.splitext(os.path.basename(lib_path))[0]
    objs = [os.path.join(OBJ_DIR, f"{tag}.{s}.o") for s in SOURCES]
    flags = compile_flags() + list(extra_flags)
    with ThreadPoolExecutor(max_workers=min(len(SOURCES), os.cpu_count() or 1)) as pool:
        jobs = [pool.submit(_run, [hipcc] + flags + ["-c", os.path.join(CSRC, s), "-o", o], verbose)
                for s, o in zip(SOURCES, objs)]
        for j in jobs:
            j.result()
    _run([hipcc, "--offload-arch=gfx950", "-fPIC", "-shared", "-o", lib_path] + list(extra_flags) + objs,
         verbose)
    if lib_path == LIB_PATH:
        # the stand-alone chip-rate measurement (not part of the library) is compiled with it so
        # that it keeps building
        _run([hipcc, "--offload-arch=gfx950", "-O3", "-o", os.path.join(OBJ_DIR, "chip_rates"),
              os.path.join(CSRC, "chip_rates.hip")], verbose)
    return lib_path


HOST_SANITIZE = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                 "-Xarch_host", "-fno-omit-frame-pointer", "-g"]


if __name__ == "__main__":
    import argparse
    ap = argparse.ArgumentParser(description=__doc__)
    ap.add_argument("--out", default=LIB_PATH, help="path of the shared library to write")
    ap.add_argument("--host-sanitize", action="store_true",
                    help="instrument the HOST code (argument checks, launchers, rollout manager) with "
                         "AddressSanitizer + UBSan; device code is built as usual.  Load the result with "
                         "COPRIS_LIB=<out> and the sanitizer runtime preloaded")
    ap.add_argument("--define", action="append", default=[], metavar="NAME",
                    help="define a preprocessor symbol (the timing probes documented in csrc/lmhead.hip); "
                         "use with --out: such a build computes wrong results by design")
    a = ap.parse_args()
    flags = (HOST_SANITIZE if a.host_sanitize else []) + ["-D" + d for d in a.define]
    print(build(verbose=True, lib_path=os.path.abspath(a.out), extra_flags=flags))
