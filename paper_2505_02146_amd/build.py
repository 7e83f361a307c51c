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


def _compile(src: str, poison: bool = False) -> str:
    obj = (OBJ / "poison" if poison else OBJ) / (src + ".o")
    cmd = ["hipcc", *FLAGS, *EXTRA_FLAGS.get(src, []), *(["-DXP_LDS_POISON"] if poison else []), "-c", str(CSRC / src), "-o", str(obj)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}{' (poison build)' if poison else ''}:\n{err}")
    return str(obj)


def _link(lib: pathlib.Path, objs, verbose: bool) -> pathlib.Path:
    r = subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", str(lib), *objs], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link of {lib.name} failed:\n" + r.stderr)
    if verbose:
        print("built", lib)
    return lib


POISONED = [s for s in SOURCES if s.startswith("xp_mfma_dl")]        # the direct-to-LDS kernels
LIB_POISON = HERE / "libxp_poison.so"


def build(verbose: bool = False) -> pathlib.Path:
    OBJ.mkdir(exist_ok=True)
    with cf.ThreadPoolExecutor(max_workers=6) as ex:
        objs = list(ex.map(_compile, SOURCES))
    return _link(LIB, objs, verbose)


def build_poison(verbose: bool = False) -> pathlib.Path:
    """libxp_poison.so: the library with -DXP_LDS_POISON in the direct-to-LDS kernels (see lds_poison in
    csrc/xp_mfma_dl.hpp); the other objects are those of build(), which must have run."""
    (OBJ / "poison").mkdir(parents=True, exist_ok=True)
    with cf.ThreadPoolExecutor(max_workers=3) as ex:
        objs = list(ex.map(lambda src: _compile(src, True), POISONED))
    return _link(LIB_POISON, objs + [str(OBJ / (s + ".o")) for s in SOURCES if s not in POISONED], verbose)


def build_all(verbose: bool = False) -> None:
    """Both libraries, their compilations side by side (the longest translation unit sets the time)."""
    (OBJ / "poison").mkdir(parents=True, exist_ok=True)
    jobs = [(s, True) for s in POISONED] + [(s, False) for s in SOURCES]           # the long ones first
    jobs.sort(key=lambda j: not j[0].startswith("xp_mfma_dl"))
    with cf.ThreadPoolExecutor(max_workers=8) as ex:
        objs = dict(zip(jobs, ex.map(lambda j: _compile(*j), jobs)))
    _link(LIB, [objs[(s, False)] for s in SOURCES], verbose)
    _link(LIB_POISON, [objs[(s, s in POISONED)] for s in SOURCES], verbose)


if __name__ == "__main__":
    build_all(verbose=True)
