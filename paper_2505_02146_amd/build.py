"""Build libxp.so (HIP kernels + C ABI) in-tree for gfx950 with hipcc."""
from __future__ import annotations

import concurrent.futures as cf
import pathlib
import subprocess

HERE = pathlib.Path(__file__).resolve().parent
CSRC = HERE / "csrc"
INCLUDE = HERE.parent / "include"
LIB = HERE / "libxp.so"
OBJ = HERE / "_build"

SOURCES = ["xp_api.hip", "xp_generic.hip", "xp_mfma_f32.hip", "xp_mfma_kc.hip", "xp_mfma_dl.hip", "xp_mfma_dl_asm.hip", "xp_mfma_dl_pair.hip", "xp_mfma_oc.hip", "xp_mfma_sk.hip", "xp_mfma_pp.hip", "xp_attention.hip", "xp_gemv.hip", "xp_tune.hip", "xp_memops.hip", "xp_conv_nchw.hip", "xp_deform_attn.hip", "xp_probe.hip", "xp_mfma_rs.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-I", str(INCLUDE), "-I", str(CSRC),
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]
# The attention kernel rescales its MFMA accumulators with vector arithmetic in every step: keep
# them in ordinary vector registers instead of moving them to and from the accumulation registers.
EXTRA_FLAGS = {"xp_attention.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"]}


def _compile(src: str) -> str:
    obj = OBJ / (src + ".o")
    cmd = ["hipcc", *FLAGS, *EXTRA_FLAGS.get(src, []), "-c", str(CSRC / src), "-o", str(obj)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    return str(obj)


def build(verbose: bool = False) -> pathlib.Path:
    OBJ.mkdir(exist_ok=True)
    with cf.ThreadPoolExecutor(max_workers=6) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", str(LIB), *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    if verbose:
        print("built", LIB)
    return LIB


def build_poison(verbose: bool = False) -> pathlib.Path:
    """libxp_poison.so: the library with -DXP_LDS_POISON in the direct-to-LDS kernels (see lds_poison in
    csrc/xp_mfma_dl.hpp); the other objects are those of build(), which must have run."""
    out = OBJ / "poison"
    out.mkdir(parents=True, exist_ok=True)
    dl = [s for s in SOURCES if s.startswith("xp_mfma_dl")]

    def one(src: str) -> str:
        obj = out / (src + ".o")
        cmd = ["hipcc", *FLAGS, "-DXP_LDS_POISON", "-c", str(CSRC / src), "-o", str(obj)]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src} (poison build):\n" + "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l))
        return str(obj)

    with cf.ThreadPoolExecutor(max_workers=3) as ex:
        objs = list(ex.map(one, dl))
    objs += [str(OBJ / (s + ".o")) for s in SOURCES if s not in dl]
    lib = HERE / "libxp_poison.so"
    r = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", str(lib), *objs], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed (poison build):\n" + r.stderr)
    if verbose:
        print("built", lib)
    return lib


if __name__ == "__main__":
    build(verbose=True)
    build_poison(verbose=True)
