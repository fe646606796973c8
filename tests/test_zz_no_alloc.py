"""The projection entry point that allocates nothing (fixed scratch buffer in device memory)
against the entry point that takes a workspace: same kernels, so the results must be
bit-identical, and both within the projection tolerance of an fp64 product.  Two calls in a
row, the second with a smaller input (the buffer keeps the first call's contents)."""
import pytest
import torch

pytestmark = pytest.mark.gpu


def _case(rows, n, k, seed):
    g = torch.Generator().manual_seed(seed)
    x = torch.randn(rows, k, generator=g, dtype=torch.float32)
    w = (torch.randn(n, k, generator=g, dtype=torch.float32) * 0.05).to(torch.bfloat16)
    return x.cuda(), w.cuda()


def test_static_scratch_entry_matches_workspace_entry():
    from paper_2410_20488_amd import binding
    lib = binding.load_library()
    cap = lib.firp_gemm_static_capacity()
    assert cap == 32 << 20
    for rows, n, k, seed in ((67, 2048, 2048, 1), (5, 520, 1032, 2)):   # the second is smaller and ragged
        assert lib.firp_gemm_workspace_bytes(rows, n, k) <= cap
        x, w = _case(rows, n, k, seed)
        want = binding.debug_gemm(x, w, 1)
        y = torch.full((rows, n), float("nan"), dtype=torch.float32, device=x.device)
        before = torch.cuda.memory_allocated()
        binding.debug_gemm_static(x, w, y)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        assert torch.equal(y, want), f"{rows}x{n}x{k}: {(y - want).abs().max().item():.3e}"
        ref = x.double() @ w.double().T
        err = (y.double() - ref).abs().max().item() / ref.std().item()
        assert err < 1e-4, err


def test_static_scratch_entry_rejects_what_does_not_fit():
    from paper_2410_20488_amd import binding
    lib = binding.load_library()
    x, w = _case(4, 8, 8, 3)
    y = torch.empty(4, 8, dtype=torch.float32, device="cuda")
    # 67 x 5120 x 5120 needs far more than the fixed buffer: refused on the host, nothing enqueued
    rc = lib.firp_debug_gemm_static(x.data_ptr(), w.data_ptr(), y.data_ptr(), 67, 5120, 5120,
                                    torch.cuda.current_stream().cuda_stream)
    assert rc == -3 and b"scratch" in lib.firp_last_error(None)
    rc = lib.firp_debug_gemm_static(None, w.data_ptr(), y.data_ptr(), 4, 8, 8, torch.cuda.current_stream().cuda_stream)
    assert rc == -1
