"""Builds libaura_fuse.so (hand-written HIP for gfx950) next to this file with hipcc."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor
from pathlib import Path

PKG = Path(__file__).resolve().parent
CSRC = PKG / "csrc"
LIB = PKG / "libaura_fuse.so"
SOURCES = ["aura_abi.hip", "project_visibility.hip", "fuse_features.hip", "fuse_tile.hip", "material_scores.hip",
           "tile_scores.hip", "knn_densify.hip", "thickness_integrate.hip", "select_views.hip", "voxel_downsample.hip", "patch_batch.hip", "estimate_normals.hip", "property_integrate.hip", "calibrate.hip", "no_alloc.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-fast-math",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function"]
# fuse_tile.hip: the product kernel asks for its tile tickets (an atomic add by one lane) long before it
# reads the answer; the compiler's wave-level rewrite of atomics would make the wave wait for the answer
# on the spot.
EXTRA_FLAGS = {"fuse_tile.hip": ["-mllvm", "-amdgpu-atomic-optimizer-strategy=None"]}


def _compile(src: str) -> Path:
    obj = CSRC / (Path(src).stem + ".o")
    cmd = [HIPCC, *FLAGS, *EXTRA_FLAGS.get(src, []), "-c", str(CSRC / src), "-o", str(obj)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{r.stdout}\n{r.stderr}")
    # the host pass warns that it does not know the packed-fp32 feature; anything else is shown
    noise = [l for l in r.stderr.splitlines() if l.strip() and "packed-fp32-ops" not in l]
    if noise:
        print("\n".join(noise))
    return obj


def build(verbose: bool = False) -> Path:
    """Compiles every kernel source for gfx950 and links the shared library.  Always recompiles."""
    with ThreadPoolExecutor(max_workers=min(len(SOURCES), os.cpu_count() or 4)) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", str(LIB), *map(str, objs)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")
    if verbose:
        print(f"built {LIB}")
    return LIB


if __name__ == "__main__":
    build(verbose=True)
