"""e2f_attn_forward_static, the form of the fused call for callers that cannot allocate: its workspace is a fixed
array inside the library.  Checked against e2f_attn_forward (same kernels, so the same bits) on two calls in a row, the
second on a smaller input, and against the size limit."""
import ctypes

import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_cuda():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2601_16622_amd import binding as B
    B.load()
    return torch


def test_static_scratch_forward_matches_the_workspace_form(torch_cuda):
    torch = torch_cuda
    from paper_2601_16622_amd import binding as B, workloads as W
    # first a box of 2 500 atoms at the benchmark's shape (tile kernel, 25 MB of the 32 MB array), then a smaller batch
    # with a partial last tile, then fp32 features through the vector-ALU kernel: each against the workspace form
    rng = np.random.default_rng(3)
    cfg = dict(L=2, C=64, H=4, B=5, lf=1, cutoff=3.5, dtype="bf16")
    cases = [W.box(2500, seed=8), W._pack(cfg, [W.dart_throw_box(rng, 333, 9.0)], rng, elements=False), W.tiny(1)]
    for wl in cases:
        P = B.Problem(wl)
        try:
            assert B.e2f_attn_workspace_bytes(P.ctx, P.N) <= B.STATIC_SCRATCH_BYTES
            P.build_cells()
            want = P.forward().clone()
            got = torch.full_like(P.out, float("nan"))
            before = torch.cuda.memory_allocated()
            P.forward_static(got)
            torch.cuda.synchronize()
            assert torch.cuda.memory_allocated() == before
            assert torch.isfinite(got).all()
            assert torch.equal(got, want), float((got - want).abs().max())
        finally:
            P.close()


def test_static_scratch_rejects_what_does_not_fit(torch_cuda):
    from paper_2601_16622_amd import binding as B, workloads as W
    wl = W.box(4000, seed=8)
    P = B.Problem(wl)
    try:
        assert B.e2f_attn_workspace_bytes(P.ctx, P.N) > B.STATIC_SCRATCH_BYTES
        P.build_cells()
        with pytest.raises(B.E2fError) as e:
            P.forward_static()
        assert e.value.code == 6 and "static scratch" in str(e.value)
    finally:
        P.close()
