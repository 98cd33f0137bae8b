"""The debug build of the library (range asserts in the kernels: select indices of Sec. 3.1 Eq. 3 against the
sketch width, LDS addresses of gathers and table copies, channel and block numbers) runs the small parity suite in
a process of its own; the session fails on any counted violation (tests/conftest.py)."""
import os
import subprocess
import sys

import pytest

import paper_2506_17255_amd as skl
from paper_2506_17255_amd import build as skl_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_the_normal_build_has_no_range_asserts():
    if "debug" in os.path.basename(skl_build.lib_path()):
        pytest.skip("running on the debug build")
    with pytest.raises(skl.SketchLinearError) as err:
        skl.sketch_linear_debug_violations()
    assert err.value.status == skl.SKL_ERR_UNSUPPORTED


@pytest.mark.gpu
@pytest.mark.skipif("debug" in os.path.basename(os.environ.get("SKETCH_LINEAR_LIB", "")), reason="already inside the debug run")
def test_parity_suite_on_the_build_with_range_asserts():
    assert os.path.exists(skl_build.DEBUG_LIB), "build it first: python -m paper_2506_17255_amd.build --debug-bounds"
    env = dict(os.environ, SKETCH_LINEAR_LIB=skl_build.DEBUG_LIB)
    res = subprocess.run([sys.executable, "-u", "-m", "pytest", "-x", "-q", "-m", "gpu", "-p", "no:cacheprovider", "--timeout", "300",
                          "--timeout-method", "thread", "tests/test_gpu_parity.py"], cwd=ROOT, env=env, capture_output=True,
                         text=True, timeout=1200)
    report = res.stdout[-3000:] + res.stderr[-2000:]
    assert res.returncode == 0, report
    assert "range asserts of the debug build: 0 violation(s)" in res.stdout, report
    assert " passed" in res.stdout


SELFTEST = """
import torch, paper_2506_17255_amd as skl
torch.zeros(1, device="cuda:0")
assert skl.sketch_linear_debug_violations()[0] == 0
skl.sketch_linear_debug_selftest(2, 3)            # in range: nothing counted
torch.cuda.synchronize()
assert skl.sketch_linear_debug_violations()[0] == 0
skl.sketch_linear_debug_selftest(5, 3)
skl.sketch_linear_debug_selftest(9, 4)
torch.cuda.synchronize()
count, first = skl.sketch_linear_debug_violations()
assert count == 2, count
assert (first["code"], first["value"], first["limit"], first["workgroup"], first["thread"]) == (7, 5, 3, 0, 0), first
print("selftest ok")
"""


@pytest.mark.gpu
def test_a_violation_is_counted_and_its_first_record_kept():
    assert os.path.exists(skl_build.DEBUG_LIB), "build it first: python -m paper_2506_17255_amd.build --debug-bounds"
    env = dict(os.environ, SKETCH_LINEAR_LIB=skl_build.DEBUG_LIB)
    res = subprocess.run([sys.executable, "-c", SELFTEST], cwd=ROOT, env=env, capture_output=True, text=True, timeout=300)
    assert res.returncode == 0 and "selftest ok" in res.stdout, res.stdout[-2000:] + res.stderr[-2000:]
