"""Build libfge.so (the C-ABI library) in-tree with hipcc for gfx950.

    python -m paper_2512_23424_amd.build [--force]

The translation units compile in parallel; the library is written next to this file so
it travels with the source tree.  Packed-fp32 instruction selection is switched off for the
device pass (the host pass prints a harmless "not a recognized feature" note)."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libfge.so")
OBJDIR = os.path.join(HERE, "_build")
UNITS = ["fge_api.hip", "fge_tiles_f32.hip", "fge_tiles_f32s.hip", "fge_tiles_bf16.hip", "fge_tiles_f16.hip", "fge_tiles_f8.hip", "fge_panel_f32.hip", "fge_generic.hip", "fge_gated.hip",
         "fge_tiles_half_bf16.hip", "fge_tiles_half_f16.hip", "fge_tiles_half_f8.hip"]
HEADERS = ["fge_device.h", "fge_epilogue.h", "fge_tile_kernel.h", "fge_panel_kernel.h", "fge_rowops.h", "fge_launch.h", "fge_tile_table.h"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++20", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _newest_source() -> float:
    files = [os.path.join(CSRC, f) for f in UNITS + HEADERS]
    files.append(os.path.join(os.path.dirname(HERE), "include", "fge.h"))
    return max(os.path.getmtime(f) for f in files)


def _compile(unit: str) -> str:
    obj = os.path.join(OBJDIR, unit.replace(".hip", ".o"))
    cmd = ["hipcc", *FLAGS, "-c", os.path.join(CSRC, unit), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {unit}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(force: bool = False) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= _newest_source():
        return LIB
    os.makedirs(OBJDIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=len(UNITS)) as ex:
        objs = list(ex.map(_compile, UNITS))
    r = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    return LIB


if __name__ == "__main__":
    print(build(force=True))
