"""The entry point that allocates nothing (cadmm_op_wgrad_noalloc: split-K partials in a static device array) against
cadmm_op_wgrad (partials in the caller's workspace): same kernels, so the results must agree bit for bit, on two calls
in a row, the second with a smaller input, which must not see anything the first left in the shared array."""
import numpy as np
import pytest

from paper_2112_09335_amd import synth

pytestmark = pytest.mark.gpu


def test_wgrad_without_allocation_matches_the_workspace_entry_point():
    import torch
    from paper_2112_09335_amd import binding
    w = synth.config(2, 0.1)                       # N = 2000, widths 500 -> 128 -> 3: the workspace covers these shapes
    s = binding.Solver.from_workload(w, 0)
    bare = binding.Solver(device=0)                # no graph, no model, no workspace
    gen = torch.Generator(device="cuda").manual_seed(5)
    try:
        for n, K, C in ((w.N, 500, 128), (777, 128, 3)):        # wide tiles with ragged edges, then smaller and narrow
            A = torch.randn(n, K, device="cuda", generator=gen)
            G = torch.randn(n, C, device="cuda", generator=gen)
            ref = s.op_wgrad(A, G)
            out = torch.full((K, C), float("nan"), device="cuda")
            got = s.op_wgrad_noalloc(A, G, out)
            torch.cuda.synchronize()
            assert torch.equal(got, ref), (n, K, C, (got - ref).abs().max().item())
            assert torch.equal(bare.op_wgrad_noalloc(A, G), ref)
            exact = A.double().T @ G.double()
            assert (got.double() - exact).abs().max().item() <= 1e-4 * exact.abs().max().item()
        # a shape beyond the static scratch is refused before anything is launched
        A = torch.zeros(256, 5120, device="cuda")
        G = torch.zeros(256, 4096, device="cuda")
        with pytest.raises(binding.CadmmError, match="static scratch"):
            bare.op_wgrad_noalloc(A, G)
    finally:
        s.close()
        bare.close()
