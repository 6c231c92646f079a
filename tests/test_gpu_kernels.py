"""GPU parity of the individual kernels (through the C ABI) against fp64 numpy / scipy on the oracle's graph."""
import numpy as np
import pytest
import scipy.sparse as sp

from oracle.graph import OracleGraph
from paper_2112_09335_amd import synth
from parity import say

pytestmark = pytest.mark.gpu

HYPER = dict(nu=1e-3, rho=1e-3, tau0=1e-3, theta0=1e-3, eta=2.0, max_backtrack=60, fista_iters=10)


@pytest.fixture(scope="module")
def ctx():
    import torch
    from paper_2112_09335_amd import binding
    w = synth.config(3, 0.03)        # N = 6000, 32 communities, degree 15: several tiles, ragged tails
    s = binding.Solver(0)
    s.build_graph(w.N, w.src, w.dst, w.M, w.comm)
    s.set_model([1030, 512, 512, 16], **HYPER)       # reserves scratch for the widest shapes below
    s.set_workspace()
    g = OracleGraph(w.N, w.src, w.dst, w.M, w.comm)
    yield s, g, torch
    s.close()


@pytest.fixture(scope="module")
def hub_ctx():
    """A graph with hub rows far beyond the split threshold (a few nodes adjacent to thousands of others),
    so that the split-row path of the aggregation (parts + ordered combine) is exercised, ragged sizes."""
    import torch
    from paper_2112_09335_amd import binding
    rng = np.random.default_rng(77)
    N, M = 5003, 5
    comm = rng.integers(0, M, size=N).astype(np.int32)
    src = [rng.integers(0, N, size=12000)]
    dst = [rng.integers(0, N, size=12000)]
    for hub, deg in ((0, 4000), (17, 1500), (N - 1, 385), (99, 384), (100, 383)):
        nb = rng.choice(N, size=deg, replace=False)
        src.append(np.full(deg, hub))
        dst.append(nb)
    src = np.concatenate(src).astype(np.int32)
    dst = np.concatenate(dst).astype(np.int32)
    s = binding.Solver(0)
    s.build_graph(N, src, dst, M, comm)
    s.set_model([300, 64, 16], **HYPER)
    s.set_workspace()
    g = OracleGraph(N, src, dst, M, comm)
    assert np.diff(g.row_ptr).max() > 3000
    yield s, g, torch
    s.close()


@pytest.mark.parametrize("width,tile", [(3, 0), (16, 0), (64, 0), (256, 0), (300, 0), (256, 32), (256, 64), (300, 128), (7, 4)])
def test_aggregate_with_hub_rows_and_column_tiles(hub_ctx, width, tile):
    s, g, torch = hub_ctx
    say("hub aggregate width", width, "tile", tile)
    rng = np.random.default_rng(width + tile)
    X = rng.standard_normal((g.N, width)).astype(np.float32)
    s.tune("spmm_tile_cols", tile)
    try:
        Y = s.op_aggregate(torch.from_numpy(X).cuda()).cpu().numpy().astype(np.float64)
        P = s.op_aggregate_segments(torch.from_numpy(X).cuda()).cpu().numpy().astype(np.float64)
    finally:
        s.tune("spmm_tile_cols", 0)
    assert rel_err(Y, g.A @ X.astype(np.float64)) < 3e-6
    S = sp.csr_matrix((g.val, g.col, g.seg_ptr), shape=(g.n_segments, g.N))
    assert rel_err(P, (S @ X.astype(np.float64))[s.get_segment_order()]) < 3e-6


def rel_err(got, ref):
    return float(np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-300))


@pytest.mark.parametrize("width", [1, 3, 7, 16, 64, 100, 128, 256, 500, 512, 1030])
def test_aggregate_matches_sparse_product(ctx, width):
    s, g, torch = ctx
    say("aggregate width", width)
    rng = np.random.default_rng(width)
    X = rng.standard_normal((g.N, width)).astype(np.float32)
    Y = s.op_aggregate(torch.from_numpy(X).cuda())
    torch.cuda.synchronize()
    ref = g.A @ X.astype(np.float64)
    assert rel_err(Y.cpu().numpy().astype(np.float64), ref) < 2e-6


def test_aggregate_is_exact_on_integers_scaled_by_the_values(ctx):
    """With X = e_j (unit columns) the result reproduces the stored values of A~ bit for bit."""
    s, g, torch = ctx
    say("aggregate unit columns")
    cols = [0, 17, g.N - 1]
    X = np.zeros((g.N, 4), np.float32)
    for k, j in enumerate(cols):
        X[j, k] = 1.0
    Y = s.op_aggregate(torch.from_numpy(X).cuda()).cpu().numpy()
    A32 = g.A.astype(np.float32).toarray() if g.N <= 8000 else None
    for k, j in enumerate(cols):
        assert np.array_equal(Y[:, k], A32[:, j])


@pytest.mark.parametrize("width", [3, 10, 16, 256])
def test_aggregate_segments_matches_per_community_products(ctx, width):
    s, g, torch = ctx
    say("aggregate_segments width", width)
    rng = np.random.default_rng(100 + width)
    V = rng.standard_normal((g.N, width)).astype(np.float32)
    P = s.op_aggregate_segments(torch.from_numpy(V).cuda()).cpu().numpy().astype(np.float64)
    # the segments of a row partition its entries, so seg_ptr is the row pointer of an n_seg x N matrix
    S = sp.csr_matrix((g.val, g.col, g.seg_ptr), shape=(g.n_segments, g.N))
    ref = (S @ V.astype(np.float64))[s.get_segment_order()]
    assert P.shape == ref.shape
    assert rel_err(P, ref) < 2e-6
    # summing a row's segments gives the full aggregation
    full = np.zeros((g.N, width))
    np.add.at(full, g.seg_row[s.get_segment_order()], P)
    assert rel_err(full, g.A @ V.astype(np.float64)) < 2e-6


@pytest.mark.parametrize("n,K,C", [(1000, 256, 256), (777, 500, 128), (300, 128, 3), (1000, 7, 64), (129, 16, 256),
                                   (4100, 512, 512), (513, 10, 256), (2000, 256, 16), (64, 64, 64), (1, 5, 2)])
def test_transform_matches_fp64_product(ctx, n, K, C):
    s, g, torch = ctx
    say("transform", n, K, C)
    rng = np.random.default_rng(n + K + C)
    A = rng.standard_normal((n, K)).astype(np.float32)
    B = rng.standard_normal((K, C)).astype(np.float32)
    out = s.op_transform(torch.from_numpy(A).cuda(), torch.from_numpy(B).cuda()).cpu().numpy().astype(np.float64)
    ref = A.astype(np.float64) @ B.astype(np.float64)
    assert rel_err(out, ref) < 1e-5


@pytest.mark.parametrize("n,K,C", [(6000, 256, 256), (5000, 500, 128), (3000, 128, 3), (6000, 512, 512), (4097, 256, 16),
                                   (100, 7, 5), (17, 300, 40)])
def test_wgrad_matches_fp64_product(ctx, n, K, C):
    s, g, torch = ctx
    say("wgrad", n, K, C)
    rng = np.random.default_rng(n + K + C + 1)
    A = rng.standard_normal((n, K)).astype(np.float32)
    G = rng.standard_normal((n, C)).astype(np.float32)
    out = s.op_wgrad(torch.from_numpy(A).cuda(), torch.from_numpy(G).cuda()).cpu().numpy().astype(np.float64)
    ref = A.astype(np.float64).T @ G.astype(np.float64)
    assert rel_err(out, ref) < 1e-5


@pytest.mark.parametrize("n,K,C", [(3000, 512, 512), (1031, 500, 200), (2000, 128, 256), (640, 37, 129)])
def test_products_agree_on_the_fp32_and_the_bf16_split_matrix_core_paths(ctx, n, K, C):
    """Results wider than 32 columns run on the bf16 matrix cores with both operands split exactly into three bf16
    parts; the fp32 MFMA kernels stay selectable.  Both must sit at fp32 rounding of the fp64 product, also for
    operands whose rows span many orders of magnitude."""
    s, g, torch = ctx
    say("split products", n, K, C)
    rng = np.random.default_rng(n * 7 + K + C)
    A = (rng.standard_normal((n, K)) * np.exp(3.0 * rng.standard_normal((n, 1)))).astype(np.float32)
    B = (rng.standard_normal((K, C)) * np.exp(2.0 * rng.standard_normal((1, C)))).astype(np.float32)
    G = (rng.standard_normal((n, C)) * np.exp(3.0 * rng.standard_normal((n, 1)))).astype(np.float32)
    ref_nn = A.astype(np.float64) @ B.astype(np.float64)
    mag_nn = np.abs(A).astype(np.float64) @ np.abs(B).astype(np.float64)
    ref_tn = A.astype(np.float64).T @ G.astype(np.float64)
    mag_tn = np.abs(A).astype(np.float64).T @ np.abs(G).astype(np.float64)
    At, Bt, Gt = (torch.from_numpy(x).cuda() for x in (A, B, G))
    try:
        for split in (0, 1):
            s.tune("gemm_split", split)
            nn = s.op_transform(At, Bt).cpu().numpy().astype(np.float64)
            tn = s.op_wgrad(At, Gt).cpu().numpy().astype(np.float64)
            assert (np.abs(nn - ref_nn) / mag_nn).max() < 2e-6, split
            assert (np.abs(tn - ref_tn) / mag_tn).max() < 2e-6, split
    finally:
        s.tune("gemm_split", 1)


def test_calibration_kernels_report_a_rate(ctx):
    s, g, torch = ctx
    assert s.op_calibrate("copy", 1 << 22, 3) > 10.0        # GB/s
    assert s.op_calibrate("update", 1 << 22, 3) > 10.0
    assert s.op_calibrate("mfma", 200, 3) > 1.0             # TFLOP/s
    assert s.op_calibrate("mfma_bf16", 200, 3) > 1.0
    assert s.op_calibrate("mfma_bf16_valu6", 200, 3) > 1.0
