"""Build libvfm.so (hand-written HIP for gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB_PATH = os.path.join(HERE, "libvfm.so")
CEILING_PATH = os.path.join(HERE, "mfma_ceiling")   # standalone matrix-pipe ceiling measurement
SOURCES = ["vfm_api.hip", "rope3d.hip", "qknorm_rope3d.hip", "attn_fwd.hip", "attn_bwd.hip", "tattn.hip", "attn_fp8.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
    # keep the compiler from forming packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
    # the direct-to-LDS load statements name m0 as clobbered; the backend accepts that and warns
    # that m0 is a reserved register at every inlined copy
    "-Wno-inline-asm",
]


def _compile(src: str, obj_dir: str, csrc: str = CSRC) -> str:
    obj = os.path.join(obj_dir, os.path.splitext(src)[0] + ".o")
    cmd = [HIPCC, *FLAGS, "-c", os.path.join(csrc, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build_lib(verbose: bool = True, csrc: str = CSRC, out: str = LIB_PATH) -> str:
    """Compile every source under `csrc` and link them into `out` (defaults: the in-tree library)."""
    obj_dir = os.path.join(HERE, "_build") if out == LIB_PATH else out + ".obj"
    os.makedirs(obj_dir, exist_ok=True)
    with ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        objs = list(ex.map(lambda s: _compile(s, obj_dir, csrc), SOURCES))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", out, *objs]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n" + res.stderr)
    if verbose:
        print(f"built {out}")
    return out


def build_ceiling_tool(verbose: bool = True, out: str = CEILING_PATH) -> str:
    """Compile the standalone MFMA-only ceiling measurement (csrc/mfma_ceiling.hip)."""
    cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Wno-unused-command-line-argument",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           os.path.join(CSRC, "mfma_ceiling.hip"), "-o", out]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed on mfma_ceiling.hip:\n" + res.stderr)
    if verbose:
        print(f"built {out}")
    return out


if __name__ == "__main__":
    build_lib()
    build_ceiling_tool()
