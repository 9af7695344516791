"""Token-tiling boundaries of the grouped GEMM, under both tile capacities (see ffn_boundary_case.py)."""
import pytest

import paper_2205_10034_amd as M
import ffn_boundary_case

pytestmark = pytest.mark.gpu


def test_tile_boundaries_default_capacity():
    assert M.moe_get_tuning(M.MOE_TUNE_GEMM_TILE_ROWS) == 0
    assert ffn_boundary_case.main() == 0


@pytest.mark.parametrize("cap", [256, 320])
def test_tile_boundaries_forced_capacity(cap):
    M.moe_set_tuning(M.MOE_TUNE_GEMM_TILE_ROWS, cap)
    try:
        assert ffn_boundary_case.main() == 0
    finally:
        M.moe_set_tuning(M.MOE_TUNE_GEMM_TILE_ROWS, 0)


@pytest.mark.parametrize("mfma", [16, 32])
def test_tile_boundaries_forced_mfma_shape(mfma):
    """The 256-row kernels with either matrix instruction (few rows per expert pick 32x32x16 by themselves)."""
    M.moe_set_tuning(M.MOE_TUNE_GEMM_TILE_ROWS, 256)
    M.moe_set_tuning(M.MOE_TUNE_GEMM_MFMA, mfma)
    try:
        assert ffn_boundary_case.main() == 0
    finally:
        M.moe_set_tuning(M.MOE_TUNE_GEMM_TILE_ROWS, 0)
        M.moe_set_tuning(M.MOE_TUNE_GEMM_MFMA, 0)
