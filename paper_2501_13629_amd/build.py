"""Build libdiffqkv.so (the HIP kernels and the C ABI) for gfx950 with hipcc, in-tree.

    python -m paper_2501_13629_amd.build        # rebuild if a source is newer than the library
    python -m paper_2501_13629_amd.build -f     # always rebuild
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor
from pathlib import Path

PKG = Path(__file__).resolve().parent
CSRC = PKG / "csrc"
INCLUDE = PKG.parent / "include"
LIB = PKG / "libdiffqkv.so"
OBJ = PKG / "_build"

SOURCES = ["api.hip", "decode_generic.hip", "decode_mfma.hip", "prefill_generic.hip", "prefill_mfma.hip", "prefill_mfma64.hip", "probe.hip", "append.hip", "topk.hip", "augq.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def stale() -> bool:
    if not LIB.exists():
        return True
    t = LIB.stat().st_mtime
    deps = [CSRC / s for s in SOURCES] + [CSRC / "kernels.h", CSRC / "prefill_tile.h", INCLUDE / "diffqkv.h", INCLUDE / "diffqkv_experimental.h", Path(__file__)]
    return any(d.stat().st_mtime > t for d in deps)


def build(force: bool = False, verbose: bool = False, extra_flags=(), out: Path | None = None) -> Path:
    """Compile and link.  `extra_flags`/`out` build a variant of the library elsewhere (experiments)."""
    variant = out is not None
    if not variant and not force and not stale():
        return LIB
    obj_dir = OBJ if not variant else Path(str(out) + ".obj")
    obj_dir.mkdir(exist_ok=True)
    hipcc = _hipcc()
    target = LIB if not variant else Path(out)

    def compile_one(src: str) -> Path:
        obj = obj_dir / (src + ".o")
        cmd = [hipcc, *HIPCC_FLAGS, *extra_flags, "-I", str(INCLUDE), "-c", str(CSRC / src), "-o", str(obj)]
        r = subprocess.run(cmd, capture_output=True, text=True)
        err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed on %s:\n%s" % (src, err))
        if verbose and err.strip():
            print(err, file=sys.stderr)
        return obj

    with ThreadPoolExecutor(min(8, len(SOURCES))) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    tmp = target.with_suffix(".so.tmp%d" % os.getpid())
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", str(tmp), *map(str, objs)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    os.replace(tmp, target)
    return target


if __name__ == "__main__":
    print(build(force="-f" in sys.argv[1:], verbose=True))
