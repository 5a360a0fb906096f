"""The big-tile kernels on small and ragged shapes.

The tile schedule sends every product below ~8 M output elements to 128 x 128 tiles, so the
layer parity cases of test_gpu_parity.py (ragged in both dimensions, short contractions,
unaligned leading dimensions, all policies, both layouts, side stream, captured graph) never
reach the 256 x 256 / 192 x 256 / 256 x 192 kernels on their own.  The library reads
ZR_FORCE_TILES once per process, so each shape runs those cases in a child process; the
element-wise bounds are the same ones (tests/parity_util.py).
"""
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

# every test that goes through the GEMM path, except the one that asserts that its product was
# split (a forced grid is never split)
CASES = ("layer_parity or average_through or output_width or extreme_kept or same_imputation or "
         "workspace_path or backward_reuses or migrated or side_stream or captured_graph")


# (shape, ring): without the ring loop the big tiles run the 64-deep two-stage loop, which the
# library still uses when a row list on the contraction axis is too long for its copy in LDS
@pytest.mark.parametrize("shape,ring", [("256", True), ("192x256", True), ("256x192", True), ("256", False),
                                        ("192x256", False)])
def test_parity_cases_on_forced_tile_shape(shape, ring):
    import torch
    if not torch.cuda.is_available():
        pytest.skip("needs a GPU")
    env = dict(os.environ, ZR_FORCE_TILES=shape)
    if not ring:
        env["ZR_NO_RING"] = "1"
    res = subprocess.run([sys.executable, "-u", "-m", "pytest", os.path.join(ROOT, "tests", "test_gpu_parity.py"), "-x", "-q",
                          "-p", "no:cacheprovider", "-k", CASES, "--timeout", "300", "--timeout-method", "thread"],
                         cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=900)
    tail = "\n".join(res.stdout.splitlines()[-25:])
    assert res.returncode == 0, tail
    assert " passed" in tail and "failed" not in tail, tail
