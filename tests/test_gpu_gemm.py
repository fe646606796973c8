"""Per-kernel parity of the projection kernels against the plain definition y = x W^T
computed on the CPU in fp64 (the oracle's matmul sub-step), through the C ABI."""
import pytest
import torch

from paper_2410_20488_amd import binding, synth

pytestmark = pytest.mark.gpu

SHAPES = [  # rows, n, K
    (7, 688, 256), (7, 256, 688), (5, 520, 256), (5, 256, 352), (1, 1024, 256),
    (4, 5120, 5120), (16, 5120, 5120), (17, 4096, 4096), (41, 4096, 11008), (44, 11008, 4096),
    (64, 5120, 5120), (67, 5120, 5120), (67, 13824, 5120), (67, 5120, 13824), (67, 32000, 5120),
    (80, 1024, 8192), (128, 5120, 5120), (129, 1280, 5120), (200, 5120, 1024), (256, 2048, 5120),
    # more than 128 rows: one pass per 256 rows, ragged K, 256 + 12 rows
    (150, 5120, 5120), (190, 4096, 11008), (256, 13824, 5120), (160, 520, 352), (268, 5120, 5120),
    # the 129..256-row kernel: n not a multiple of its 256-row tile or of 16, an odd number of stages, one stage
    (192, 1000, 512), (255, 4100, 320), (130, 256, 64), (256, 260, 8192),
    # shapes whose plan takes that kernel's 192-row tiles (the 34B-shaped gate|up matrix among them)
    (256, 44032, 8192), (256, 1344, 1024), (180, 2112, 2048),
]


def _inputs(rows, n, K, dtype):
    dev = torch.device("cuda:0")
    x = synth.normal_tensor(7, 900 + rows, (rows, K), 1.0, torch.float32, dev)
    w = synth.normal_tensor(7, 901 + n % 97, (n, K), 0.02, dtype, dev)
    return x, w


@pytest.mark.parametrize("rows,n,K", SHAPES)
def test_mfma_projection_matches_fp64_matmul(rows, n, K):
    x, w = _inputs(rows, n, K, torch.bfloat16)
    y = binding.debug_gemm(x, w, kind=1).cpu().double()
    ref = x.cpu().double() @ w.cpu().double().T
    err = float((y - ref).abs().max() / ref.std())
    # two bf16 planes carry 16 mantissa bits of x: rounding error per product <= 2^-17 |x||w|
    assert err < 2e-4, err


@pytest.mark.parametrize("rows,n,K,dtype", [(7, 688, 256, torch.float32), (67, 1024, 688, torch.float32),
                                            (130, 520, 352, torch.bfloat16), (3, 1000, 100, torch.float32),
                                            # the one-wave-per-column kernel's range ends at 16 rows
                                            (16, 1024, 256, torch.float32), (17, 256, 256, torch.float32),
                                            (5, 520, 352, torch.bfloat16), (1, 4, 8, torch.float32),
                                            (4, 1024, 2052, torch.float32), (11, 36, 1028, torch.bfloat16)])
def test_plain_projection_matches_fp64_matmul(rows, n, K, dtype):
    x, w = _inputs(rows, n, K, dtype)
    y = binding.debug_gemm(x, w, kind=0).cpu().double()
    ref = x.cpu().double() @ w.cpu().double().T
    assert float((y - ref).abs().max() / ref.std()) < 2e-5


def _random_shapes(count, seed):
    """Seeded shapes over everything the MFMA kernels take: any row count up to 300, n a multiple of
    4, K a multiple of 8 (a quarter of them multiples of 64, which the kernel for 129..256 rows needs)."""
    g = torch.Generator().manual_seed(seed)
    out = []
    for i in range(count):
        rows = int(torch.randint(1, 301, (1,), generator=g))
        n = 4 * int(torch.randint(1, 700, (1,), generator=g))
        K = 64 * int(torch.randint(1, 40, (1,), generator=g)) if i % 4 else 8 * int(torch.randint(1, 300, (1,), generator=g))
        out.append((rows, n, K))
    return out


@pytest.mark.parametrize("rows,n,K", _random_shapes(48, 20488))
def test_mfma_projection_random_shapes(rows, n, K):
    x, w = _inputs(rows, n, K, torch.bfloat16)
    y = binding.debug_gemm(x, w, kind=1).cpu().double()
    ref = x.cpu().double() @ w.cpu().double().T
    assert float((y - ref).abs().max() / ref.std()) < 2e-4


@pytest.mark.parametrize("rows,n,K,repeats", [(256, 44032, 8192, 300), (200, 27648, 5120, 300), (67, 27648, 5120, 200),
                                             (256, 8192, 22016, 200)])   # an odd number of stages per workgroup
def test_projection_is_bit_repeatable(rows, n, K, repeats):
    """The kernels are deterministic (fixed summation order, no atomics): every launch on the same
    operands must give the same bits.  Hundreds of launches of the largest shapes - some 10^8 wave-level
    loads into LDS for the 256-row one - would show a missed wait or hazard as a rare mismatch."""
    x, w = _inputs(rows, n, K, torch.bfloat16)
    first = binding.debug_gemm(x, w, kind=1)
    bad = 0
    for _ in range(repeats):
        bad += int(not torch.equal(binding.debug_gemm(x, w, kind=1), first))
    assert bad == 0, f"{bad} of {repeats} launches differ from the first"
