"""Every kernel strides by its grid size, but a grid is smaller than the work only for lists beyond 2^32
work-items (17 G elements), which no test can hold.  SWIFT_MAX_GRID caps the grids instead: the same calls in a
process with 97 workgroups per launch must leave the bits of a process with ordinary grids (whose results the
other tests hold against the oracle)."""
import os
import subprocess
import sys

import numpy as np
import pytest

pytestmark = pytest.mark.gpu
HERE = os.path.dirname(os.path.abspath(__file__))


def _child(tmp_path, name, max_grid):
    out = str(tmp_path / name)
    env = dict(os.environ)
    env.pop("SWIFT_MAX_GRID", None)
    if max_grid:
        env["SWIFT_MAX_GRID"] = str(max_grid)
    done = subprocess.run([sys.executable, os.path.join(HERE, "capped_grid_child.py"), out], env=env,
                          capture_output=True, text=True, timeout=300)
    assert done.returncode == 0, done.stderr[-2000:]
    return np.load(out)


def test_capped_grids_leave_the_same_bits(tmp_path):
    ref = _child(tmp_path, "ref.npz", 0)
    cap = _child(tmp_path, "cap.npz", 97)
    assert sorted(ref.files) == sorted(cap.files) and len(ref.files) > 100
    for key in ref.files:
        a, b = ref[key], cap[key]
        assert a.shape == b.shape and a.dtype == b.dtype, key
        assert np.array_equal(a.view(np.uint8), b.view(np.uint8)), key
    # the runs did something: a step moved the parameters
    assert not np.array_equal(ref["adamw_step_x0"], ref["adamw_undo_x0"])
