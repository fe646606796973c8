"""Host-side checks of the projection launch plan (no GPU): the plan must cover K and n exactly
once, keep one workgroup per CU where the shape allows it, and choose the kernel for 129..256
rows only for shapes that kernel takes."""
import itertools

import pytest

from paper_2410_20488_amd import binding

SHAPES = {  # the projection matrices of the LLaMA-2-shaped workloads: q|k|v, o, gate|up, down, lm-head
    "7b": [(12288, 4096), (4096, 4096), (22016, 4096), (4096, 11008), (32000, 4096)],
    "13b": [(15360, 5120), (5120, 5120), (27648, 5120), (5120, 13824), (32000, 5120)],
    "34b": [(10240, 8192), (8192, 8192), (44032, 8192), (8192, 22016), (32000, 8192)],
    "small": [(768, 256), (256, 256), (1376, 256), (256, 688), (1024, 256), (520, 352), (1000, 104)],
}
ROWS = [1, 3, 7, 16, 44, 64, 67, 100, 128, 129, 160, 192, 200, 256, 268, 400]


@pytest.mark.parametrize("rows,shape", list(itertools.product(ROWS, [s for v in SHAPES.values() for s in v])))
def test_plan_covers_the_matrix(rows, shape):
    n, K = shape
    p = binding.gemm_plan(rows, n, K)
    S, kp, nw, grid, rb = (p[k] for k in ("splits", "k_per_split", "waves", "grid", "row_block"))
    assert 1 <= S <= 16 and 2 <= nw <= 8
    assert kp % 64 == 0 and S * kp >= K                 # the splits cover K in whole 64-column stages
    assert (S - 1) * kp < K or S == 1 or K <= 64 * S    # and no split but the last few is empty by construction
    tiles = -(-n // (32 * nw))
    assert grid == tiles * S                            # every 32*nw-row tile of W once per split
    if rows > 128 and K % 64 == 0:
        assert rb == 256 and nw in (6, 8)               # the kernel for 129..256 rows: 192- or 256-row tiles of W
    else:
        assert rb == 128
    stages = -(-K // 64)
    if S > 1:
        assert stages // S >= 4                         # no split shorter than four stages


@pytest.mark.parametrize("model", ["7b", "13b", "34b"])
@pytest.mark.parametrize("rows", [1, 44, 64, 67, 128, 256])
def test_one_workgroup_per_cu_and_most_cus_busy(model, rows):
    """At the model shapes the plan keeps every launch within one workgroup per CU (256) and at
    least two thirds of the CUs busy."""
    for n, K in SHAPES[model]:
        p = binding.gemm_plan(rows, n, K)
        assert 170 <= p["grid"] <= 256, (n, K, p)


def test_few_waves_are_not_paired_with_many_activation_tiles():
    """Two waves cannot keep a CU's memory pipeline busy while it re-reads a tall activation
    tile: from 33 rows on a workgroup has at least three waves, from 49 rows at least four."""
    for n, K in SHAPES["7b"] + SHAPES["13b"]:
        assert binding.gemm_plan(48, n, K)["waves"] >= 3
        for rows in (49, 67, 128):
            assert binding.gemm_plan(rows, n, K)["waves"] >= 4


def test_rejected_shapes():
    for rows, n, K in [(0, 256, 256), (4, 254, 256), (4, 256, 100), (4, 2, 256)]:
        with pytest.raises(binding.FirpError):
            binding.gemm_plan(rows, n, K)
