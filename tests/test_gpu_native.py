"""The library driven from a plain C program, without Python or PyTorch in the process
(so with the HIP runtime of the ROCm installation, not the one PyTorch bundles): every
primitive and data path against the C oracle.  The program is built by build()."""
import os
import subprocess

import pytest

from gpu_util import require_gpu

pytestmark = pytest.mark.gpu

EXE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "native", "gpu_native")


@pytest.mark.parametrize("sync", ["memops", "event", "host"])
def test_native_c_program(sync):
    require_gpu()
    if not os.path.exists(EXE):
        # normally built by build(); one gcc call on a C file if the tree arrived without it
        import sys
        sys.path.insert(0, os.path.dirname(EXE))
        import build_native
        build_native.build_native_check(verbose=False)
    rv = subprocess.run([EXE, sync], capture_output=True, text=True, timeout=120)
    assert rv.returncode == 0, rv.stdout[-2000:] + rv.stderr[-2000:]
    assert "native ok" in rv.stdout and f"ordering: {sync}" in rv.stdout
    assert rv.stdout.count(": ok") == 12 and "probe: workgroup 0 ran" in rv.stdout
