"""Builds libcsat.so (the HIP kernels and their C ABI) for gfx950 with hipcc, in-tree.

The library is a handful of translation units (the C ABI with the small kernels, and one unit per
instantiation group of the two large kernel families) compiled in parallel and linked into one shared
object.  build() compiles everything, every time; build(incremental=True) recompiles only the units whose
sources or flags changed since their object file was written (for the edit-compile loop)."""
import concurrent.futures
import glob
import hashlib
import os
import shutil
import subprocess

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ_DIR = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libcsat.so")
HEADERS = sorted(glob.glob(os.path.join(CSRC, "*.h"))) + [os.path.join(ROOT, "include", "csat.h")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed fp32 instructions are kept out of the generated code on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]

# (object name, source file, extra defines)
UNITS = [("csat", "csat.hip", [])]
UNITS += [(f"ista_fused_mt{mt}", "csat_tu_ista_fused.hip", [f"-DCSAT_TU_MT={mt}"]) for mt in range(1, 17)]
UNITS += [(f"attention_{'bf16' if b else 'f32'}_z{z}", "csat_tu_attention.hip", [f"-DCSAT_TU_BF16={b}", f"-DCSAT_TU_Z={z}"])
          for b in (1, 0) for z in ((0, 1, 2, 3) if b else (0, 1))]
SOURCES = sorted({os.path.join(CSRC, src) for _, src, _ in UNITS})


def _hipcc() -> str:
    return shutil.which("hipcc") or "/opt/rocm/bin/hipcc"


def _compile(unit, incremental):
    name, src, defines = unit
    obj = os.path.join(OBJ_DIR, name + ".o")
    cmd = [_hipcc(), *HIPCC_FLAGS, *defines, "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-c",
           os.path.join(CSRC, src), "-o", obj]
    stamp = obj + ".cmd"
    key = hashlib.sha256(" ".join(cmd).encode()).hexdigest()
    if incremental and os.path.exists(obj) and os.path.exists(stamp) and open(stamp).read() == key:
        t = os.path.getmtime(obj)
        if all(os.path.getmtime(p) <= t for p in HEADERS + [os.path.join(CSRC, src)]):
            return obj, None
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        return obj, f"hipcc failed on {src} {' '.join(defines)}:\n{res.stdout}{res.stderr}"
    with open(stamp, "w") as f:
        f.write(key)
    return obj, None


def build(verbose: bool = False, incremental: bool = False, jobs: int = 0) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    jobs = jobs or min(8, os.cpu_count() or 1, len(UNITS))
    with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as pool:
        results = list(pool.map(lambda u: _compile(u, incremental), UNITS))
    errors = [e for _, e in results if e]
    if errors:
        raise RuntimeError("\n".join(errors))
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", *[o for o, _ in results], "-o", LIB]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n" + res.stdout + res.stderr)
    if verbose:
        print(f"{len(UNITS)} translation units -> {LIB}")
    return LIB


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(p) > t for p in SOURCES + HEADERS)


if __name__ == "__main__":
    import sys
    print(build(verbose=True, incremental="--incremental" in sys.argv))
