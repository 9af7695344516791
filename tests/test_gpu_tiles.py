"""Token-tiling boundaries of the grouped GEMM, under both tile capacities (see ffn_boundary_case.py)."""
import os
import subprocess
import sys

import pytest

import ffn_boundary_case

pytestmark = pytest.mark.gpu
HERE = os.path.dirname(os.path.abspath(__file__))


def test_tile_boundaries_default_capacity():
    assert ffn_boundary_case.main() == 0


@pytest.mark.parametrize("cap", ["256", "320"])
def test_tile_boundaries_forced_capacity(cap):
    env = dict(os.environ, MOESYS_GEMM_TOK=cap)
    r = subprocess.run([sys.executable, os.path.join(HERE, "ffn_boundary_case.py")], env=env, capture_output=True,
                       text=True, timeout=300)
    print(r.stdout[-3000:], r.stderr[-3000:], flush=True)
    assert r.returncode == 0
