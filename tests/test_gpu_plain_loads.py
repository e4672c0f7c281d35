"""The kernels with hand-placed loads against a build of the same sources with ordinary loads.

The k-split, tile and small-block kernels issue their loads from inline assembly and place the waits
themselves; the compiler does not know that such a register is still being filled, so a copy or a spill of
one before its wait would carry garbage.  The build refuses spills; copies are caught here: the checking
build (-DBSR_PLAIN_LOADS: the same loads through builtins and plain pointers, waits placed by the compiler)
does the same arithmetic in the same order, so every result must agree bit for bit."""
import os
import subprocess
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.gpu
def test_hand_placed_loads_agree_with_ordinary_loads(tmp_path, oracle_mod):
    import paper_2007_13055_amd.binding as binding
    from paper_2007_13055_amd import build as hip_build
    import plain_loads_cases as plc
    from gpu_util import check
    assert os.path.exists(hip_build.LIB_PLAIN), "the checking build is missing: python -m paper_2007_13055_amd.build"
    assert os.path.abspath(binding.library_path()) == os.path.abspath(hip_build.LIB)
    mine = plc.run_cases()
    out = tmp_path / "plain.npz"
    r = subprocess.run([sys.executable, "-u", os.path.join(ROOT, "tests", "plain_loads_cases.py"), hip_build.LIB_PLAIN, str(out)],
                       capture_output=True, text=True, timeout=600, cwd=ROOT)
    assert r.returncode == 0, r.stdout + r.stderr
    assert os.path.abspath(hip_build.LIB_PLAIN) in r.stdout
    plain = np.load(out)
    assert sorted(plain.files) == sorted(mine)
    for name, tune, p in plc.cases():
        assert np.array_equal(mine[name], plain[name]), f"{name}: the two builds differ"
        Yo, So = oracle_mod.bsr_spmm(p.X, p.block_data, p.block_indices, p.index_pointer, p.n)
        check(mine[name], Yo, So, p.tau, name, out_dtype=p.out_dtype)
