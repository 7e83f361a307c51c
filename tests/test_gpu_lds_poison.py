"""The direct-to-LDS kernels once more in the LDS-poison debug build (libxp_poison.so, -DXP_LDS_POISON): every ring slot
is filled with NaNs right before the load that refills it is issued, so a slot that is refilled while another wave
still reads it -- a race that the ordinary build survives almost every time, the old data being still in place --
gives NaNs here every time.  The parity tests of those kernels (every variant forced in turn, whole-tile and ragged
shapes, the convolution cases, the full-size workloads) run again in a child process that loads that build."""
import os
import pathlib
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = pathlib.Path(__file__).resolve().parent.parent
POISON = ROOT / "paper_2505_02146_amd" / "libxp_poison.so"

CHILD = """
import sys
import pytest
from paper_2505_02146_amd import xp
assert xp.LIB_PATH.name == "libxp_poison.so", xp.LIB_PATH
sys.exit(pytest.main(["-x", "-q", "-m", "gpu", "-p", "no:cacheprovider", *sys.argv[1:]]))
"""

SELECTIONS = {
    "gemm": ["tests/test_gpu_parity.py", "-k",
             "(test_gemm_shapes_all_variants and (bf16 or i8) and row-col) or test_gemm_whole_tiles_with_alpha"],
    "conv": ["tests/test_gpu_parity.py", "-k", "test_conv_cases and bf16"],
    "workloads": ["tests/test_gpu_workloads.py", "-k", "bf16_4096 or i8_4096 or conv_bf16_56 or same_bits"],
}


@pytest.mark.parametrize("which", list(SELECTIONS))
def test_parity_with_poisoned_ring_slots(which):
    assert POISON.exists(), "libxp_poison.so is missing: run paper_2505_02146_amd/build.py"
    env = dict(os.environ, XP_LIBRARY=str(POISON))
    r = subprocess.run([sys.executable, "-u", "-c", CHILD, *SELECTIONS[which]], cwd=ROOT, env=env, capture_output=True,
                       text=True, timeout=600)
    tail = "\n".join((r.stdout + r.stderr).splitlines()[-25:])
    assert r.returncode == 0, tail
    assert " passed" in r.stdout and "no tests ran" not in r.stdout, tail
