"""No result of the library may depend on the order in which workgroups run (no float atomics, no
hand-over between workgroups that depends on who comes first).  A second build of the library
walks every grid backwards (workgroup i does the work of workgroup n-1-i); every entry point is
run on the same seeded inputs with both builds and all outputs must be bit-identical."""
import os
import subprocess
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu
HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
REVERSED = os.path.join(ROOT, "paper_2505_19602_amd", "libscalekv_reversed_order.so")


@pytest.mark.skipif(not os.path.exists(REVERSED),
                    reason="build it with: python -m paper_2505_19602_amd.build --variant reversed_order")
def test_outputs_do_not_depend_on_the_order_of_workgroups(tmp_path):
    sys.path.insert(0, HERE)
    try:
        import wg_order_worker
    finally:
        sys.path.remove(HERE)
    plain = wg_order_worker.run_all()
    path = str(tmp_path / "reversed.npz")
    env = dict(os.environ, SCALEKV_LIBRARY=REVERSED, PYTHONPATH=ROOT + os.pathsep + os.environ.get("PYTHONPATH", ""))
    print("workgroup order: child process with the reversed build", flush=True)
    res = subprocess.run([sys.executable, "-u", os.path.join(HERE, "wg_order_worker.py"), path], env=env, cwd=ROOT,
                         capture_output=True, text=True, timeout=600)
    assert res.returncode == 0, f"worker failed:\n{res.stdout[-2000:]}\n{res.stderr[-4000:]}"
    rev = np.load(path)
    assert sorted(rev.files) == sorted(plain), "the two runs produced different sets of outputs"
    assert str(plain.pop("library")) == "libscalekv.so" and str(rev["library"]) == os.path.basename(REVERSED)
    for name in sorted(plain):
        a, b = plain[name], rev[name]
        assert a.shape == b.shape and a.dtype == b.dtype, name
        assert a.tobytes() == b.tobytes(), f"{name} differs between the plain and the reversed build"
