"""Builds libvcnn.so (HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor
from pathlib import Path

PKG = Path(__file__).resolve().parent
CSRC = PKG / "csrc"
LIB = PKG / "libvcnn.so"
# measurement aids of the benchmark (register-only MFMA loop, plain copy): a shared object of their own
AID_SRC = PKG / "benchaid" / "benchaid.hip"
AID_LIB = PKG / "libvcnn_benchaid.so"
OBJ_DIR = PKG / "_build"
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def sources():
    return sorted(CSRC.glob("*.hip"))


def _fresh(obj: Path, src: Path) -> bool:
    """True if obj is newer than its source and every header beside it."""
    if not obj.exists():
        return False
    t = obj.stat().st_mtime
    deps = [src, *CSRC.glob("*.h"), PKG.parent / "include" / "vcnn.h", Path(__file__)]
    return all(d.stat().st_mtime < t for d in deps)


def _compile(src: Path, incremental: bool = False) -> Path:
    obj = OBJ_DIR / (src.stem + ".o")
    if incremental and _fresh(obj, src):
        return obj
    cmd = [HIPCC, *FLAGS, "-c", str(src), "-o", str(obj)]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src.name}:\n{res.stdout}\n{res.stderr}")
    warn = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l and l.strip())
    if "warning" in warn:
        sys.stderr.write(warn + "\n")
    return obj


def build(verbose: bool = False, incremental: bool = False) -> Path:
    """Compiles every HIP source and links the shared libraries.  Recompiles everything unless `incremental`
    (then only sources newer than their objects; a development convenience)."""
    OBJ_DIR.mkdir(exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(sources()))) as ex:
        objs = list(ex.map(lambda s: _compile(s, incremental), sources()))
    tmp = LIB.with_suffix(f".so.tmp{os.getpid()}")
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", str(tmp), *map(str, objs)]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"link failed:\n{res.stdout}\n{res.stderr}")
    os.replace(tmp, LIB)
    tmp = AID_LIB.with_suffix(f".so.tmp{os.getpid()}")
    res = subprocess.run([HIPCC, *FLAGS, "-shared", "-o", str(tmp), str(AID_SRC)], capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed for {AID_SRC.name}:\n{res.stdout}\n{res.stderr}")
    os.replace(tmp, AID_LIB)
    if verbose:
        print(f"built {LIB} and {AID_LIB.name}")
    return LIB


if __name__ == "__main__":
    build(verbose=True, incremental="--incremental" in sys.argv[1:])
