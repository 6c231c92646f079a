"""Parity at the full size of the benchmark workload (2,000,000-node power-law SBM, the launch
configuration bench.py times): the graph bit for bit, kernels on sampled outputs, the readout against the
oracle's full-graph forms on the library's own state, and properties of one more iteration that hold at
any size (dual step identity, last-layer rows, sufficient decrease of every W step and of sampled Z steps)."""
import time

import numpy as np
import pytest

from oracle.admm import AdmmOracle, fista_rows, inner, relu, sqnorm
from oracle.graph import OracleGraph
from paper_2112_09335_amd import synth
from parity import REL, say

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def full():
    import torch
    from paper_2112_09335_amd import binding
    t0 = time.time()
    w = synth.config(4)
    say(f"generated {w.name}: N={w.N} E={w.E} in {time.time() - t0:.0f} s")
    t0 = time.time()
    s = binding.Solver.from_workload(w, 0)
    say(f"library ready in {time.time() - t0:.0f} s")
    t0 = time.time()
    g = OracleGraph(w.N, w.src, w.dst, w.M, w.comm, split=False)
    say(f"oracle graph in {time.time() - t0:.0f} s")
    yield w, s, g, torch
    s.close()


def relmax(got, ref):
    return float(np.abs(np.asarray(got, np.float64) - ref).max() / max(np.abs(ref).max(), 1e-300))


def test_graph_is_bit_exact_at_full_size(full):
    w, s, g, torch = full
    gg = s.get_graph()
    assert s.graph_sizes() == (g.nnz, g.n_segments, g.n_halo_rows)
    assert np.array_equal(gg["perm"], g.perm)
    assert np.array_equal(gg["row_ptr"], g.row_ptr)
    assert np.array_equal(gg["col"], g.col)
    assert np.array_equal(gg["val"].view(np.uint32), g.val.astype(np.float32).view(np.uint32))
    assert np.array_equal(gg["seg_ptr"], g.seg_ptr)
    assert np.array_equal(gg["seg_row"], g.seg_row)
    assert np.array_equal(gg["seg_comm"], g.seg_comm)
    assert np.array_equal(gg["comm_row_ptr"], g.comm_row_ptr)
    assert np.array_equal(gg["neighbour"], g.neighbour)


def test_kernels_on_sampled_outputs_at_full_size(full):
    w, s, g, torch = full
    rng = np.random.default_rng(0)
    deg = np.diff(g.row_ptr)
    rows = np.unique(np.concatenate([rng.integers(0, g.N, 400), np.argsort(-deg)[:20], [0, g.N - 1]]))
    order = s.get_segment_order()
    for width in (256, 16):
        say("full-size aggregate width", width)
        X = rng.standard_normal((g.N, width)).astype(np.float32)
        Xd = torch.from_numpy(X).cuda()
        Y = s.op_aggregate(Xd)[torch.from_numpy(rows).cuda()].cpu().numpy()
        ref = g.A[rows, :] @ X.astype(np.float64)
        assert relmax(Y, ref) < 3e-6
        if width == 16:
            segs = np.unique(np.concatenate([rng.integers(0, g.n_segments, 400),
                                             np.flatnonzero(np.isin(g.seg_row[order], np.argsort(-deg)[:5]))[:200]]))
            P = s.op_aggregate_segments(Xd)[torch.from_numpy(segs).cuda()].cpu().numpy()
            X64 = X.astype(np.float64)
            for k, j in enumerate(segs):
                sidx = order[j]
                lo, hi = g.seg_ptr[sidx], g.seg_ptr[sidx + 1]
                refrow = g.val[lo:hi] @ X64[g.col[lo:hi]]
                assert np.abs(P[k] - refrow).max() <= 3e-6 * max(np.abs(refrow).max(), 1.0)
        del Xd
    say("full-size transform / wgrad")
    A = rng.standard_normal((g.N, 128)).astype(np.float32)
    B = rng.standard_normal((128, 256)).astype(np.float32)
    G = rng.standard_normal((g.N, 16)).astype(np.float32)
    Ad = torch.from_numpy(A).cuda()
    out = s.op_transform(Ad, torch.from_numpy(B).cuda())[torch.from_numpy(rows).cuda()].cpu().numpy()
    assert relmax(out, A[rows].astype(np.float64) @ B.astype(np.float64)) < 1e-5
    wg = s.op_wgrad(Ad, torch.from_numpy(G).cuda()).cpu().numpy()
    assert relmax(wg, A.astype(np.float64).T @ G.astype(np.float64)) < 1e-5


def test_readout_and_iteration_properties_at_full_size(full):
    w, s, g, torch = full
    h = w.hyper
    o = AdmmOracle(g, w.dims, nu=h["nu"], rho=h["rho"], tau0=h["tau0"], theta0=h["theta0"], eta=h["eta"],
                   max_backtrack=h["max_backtrack"], fista_iters=h["fista_iters"], risk=h["risk"])
    o.set_data(w.X, w.labels)
    L = w.L

    def pull():
        """The library's state as fp64 arrays in the oracle's (internal) node order."""
        W = [None] + [s.get_W(l).astype(np.float64) for l in range(1, L + 1)]
        Z = [o.Z[0]] + [g.to_new(s.get_Z(l).astype(np.float64)) for l in range(1, L + 1)]
        U = g.to_new(s.get_U().astype(np.float64))
        return W, Z, U

    s.run(3)
    W0, Z0, U0 = pull()
    say("full-size readout vs oracle full-graph forms")
    sg = s.eval()
    so = o.stats_full_graph(W0, Z0, U0)
    for key in ("objective", "lagrangian", "risk", "primal_res"):
        assert abs(sg[key] - so[key]) <= REL * abs(so[key]), (key, sg[key], so[key])
    assert abs(sg["layer_penalty"][0] - so["layer_penalty"][0]) <= REL * so["layer_penalty"][0]

    tau_before, theta_before, _, _ = s.get_steps()
    s.run(1)
    W1, Z1, U1 = pull()
    tau, theta, trials, sq = s.get_steps()
    assert s.eval()["status"] == 0

    say("dual step identity (Eq. 2) on every row")
    TL = g.A @ (Z0[L - 1] @ W1[L])
    want = U0 + o.rho * (Z0[L] - TL)
    assert np.abs(U1 - want).max() <= REL * np.abs(want).max()

    say("last layer: sampled rows against the oracle's FISTA")
    rng = np.random.default_rng(1)
    rows = rng.integers(0, g.N, 2000)
    zref = fista_rows(Z0[L][rows], TL[rows], U0[rows], o.Y[rows], o.labelled[rows], o.rho, o.J, o.risk)
    assert np.abs(Z1[L][rows] - zref).max() <= REL * np.abs(zref).max()

    say("every W step satisfies the condition on tau, with the smallest exponent")
    for l in range(1, L + 1):
        dW = W1[l] - W0[l]
        t = tau[l - 1]
        if trials[l - 1] == 0:
            assert not dW.any()
            continue
        phi0 = o.phi_full_graph(l, W0[l], Z0[l - 1], Z0[l], U0)
        phi1 = o.phi_full_graph(l, W1[l], Z0[l - 1], Z0[l], U0)
        gsq = t * t * sqnorm(dW)                        # ||grad||^2, since dW = -grad/tau
        assert abs(gsq - sq[l - 1]) <= 1e-4 * sq[l - 1]
        assert phi1 <= phi0 - gsq / (2 * t) + 1e-6 * abs(phi0)
        assert t >= tau_before[l - 1]
        if trials[l - 1] > 1:                            # the candidate before the accepted one fails
            tp = t / o.eta
            Wp = W0[l] - dW * (t / tp)
            assert o.phi_full_graph(l, Wp, Z0[l - 1], Z0[l], U0) > phi0 - gsq / (2 * tp)

    say("sampled Z steps lower Eq. 1 by at least ||grad||^2 / (2 theta)")
    base = o.stats_full_graph(W1, Z0, U0)["lagrangian"] - o.risk_value(Z0[L], o.Y, o.labelled)
    for m in (0, 17, 63):
        r = g.rows(m)
        th = theta[m]
        dZ = Z1[1][r] - Z0[1][r]
        if trials[L + m] == 0:
            assert not dZ.any()
            continue
        Zm = [z for z in Z0]
        Zm[1] = Z0[1].copy()
        Zm[1][r] = Z1[1][r]
        val = o.stats_full_graph(W1, Zm, U0)["lagrangian"] - o.risk_value(Z0[L], o.Y, o.labelled)
        gsq = th * th * sqnorm(dZ)
        assert abs(gsq - sq[L + m]) <= 1e-4 * sq[L + m]
        assert val <= base - gsq / (2 * th) + 1e-7 * abs(base), (m, val, base, gsq / (2 * th))


def test_last_layer_with_backtracking_at_full_size(full):
    """fista_mode 1 on the 2,000,000-node workload: the blocks Z_{L,m} of sampled communities against the oracle's
    block solver run on the library's own state (the oracle handles one community of 31,000 rows in a moment), with
    the accepted L and the trial count of those communities equal, and Eq. 2 on every row."""
    from paper_2112_09335_amd import binding
    w, _, g, torch = full
    w1 = synth.Workload(w.name, w.N, w.M, w.src, w.dst, w.comm, w.X, w.labels, list(w.dims), w.W0, w.iters,
                        dict(w.hyper, fista_mode=1))
    s = binding.Solver.from_workload(w1, 0)
    try:
        h = w1.hyper
        o = AdmmOracle(g, w.dims, nu=h["nu"], rho=h["rho"], tau0=h["tau0"], theta0=h["theta0"], eta=h["eta"],
                       max_backtrack=h["max_backtrack"], fista_iters=h["fista_iters"], risk=h["risk"], fista_mode=1)
        o.set_data(w.X, w.labels)
        L = w.L
        s.run(2)
        ZL0 = g.to_new(s.get_Z(L).astype(np.float64))
        Zp0 = g.to_new(s.get_Z(L - 1).astype(np.float64))
        U0 = g.to_new(s.get_U().astype(np.float64))
        s.run(1)
        assert s.eval()["status"] == 0
        WL1 = s.get_W(L).astype(np.float64)
        ZL1 = g.to_new(s.get_Z(L).astype(np.float64))
        U1 = g.to_new(s.get_U().astype(np.float64))
        TL = g.A @ (Zp0 @ WL1)
        say("dual step identity (Eq. 2) with the block solver in place")
        want = U0 + o.rho * (ZL0 - TL)
        assert np.abs(U1 - want).max() <= REL * np.abs(want).max()
        Lgpu, trials_gpu = s.get_fista()
        for m in (0, 23, 63):
            say("community", m, "against the oracle's block solver")
            r = g.rows(m)
            zref = o.fista_block_backtracking(m, ZL0[r], TL[r], U0[r], o.J)
            assert np.abs(ZL1[r] - zref).max() <= REL * np.abs(zref).max(), m
            assert Lgpu[m] == o.fista_L[m] and trials_gpu[m] == o.fista_trials[m], (m, Lgpu[m], o.fista_L[m],
                                                                                      trials_gpu[m], o.fista_trials[m])
            assert o.rho <= Lgpu[m] <= o.eta * (o.rho + 0.5)      # cross-entropy: curvature at most rho + 1/2
    finally:
        s.close()


@pytest.mark.parametrize("index", [3, 5])
def test_readout_and_dual_step_at_full_size_of_the_other_large_configs(index):
    """Configs 3 (three layers, 32 communities) and 5 (eight layers of 512): after a few iterations the library's
    readout must equal the oracle's full-graph forms evaluated on the library's own state, the last-layer step
    must match the oracle's row solver and the dual step must satisfy Eq. 2 on every row."""
    import torch  # noqa: F401
    from paper_2112_09335_amd import binding
    w = synth.config(index)
    say(f"config {index}: N={w.N} E={w.E} dims={w.dims}")
    s = binding.Solver.from_workload(w, 0)
    g = OracleGraph(w.N, w.src, w.dst, w.M, w.comm, split=False)
    h = w.hyper
    o = AdmmOracle(g, w.dims, nu=h["nu"], rho=h["rho"], tau0=h["tau0"], theta0=h["theta0"], eta=h["eta"],
                   max_backtrack=h["max_backtrack"], fista_iters=h["fista_iters"], risk=h["risk"])
    o.set_data(w.X, w.labels)
    L = w.L

    def pull():
        W = [None] + [s.get_W(l).astype(np.float64) for l in range(1, L + 1)]
        Z = [o.Z[0]] + [g.to_new(s.get_Z(l).astype(np.float64)) for l in range(1, L + 1)]
        return W, Z, g.to_new(s.get_U().astype(np.float64))

    s.run(4)
    W0, Z0, U0 = pull()
    sg = s.eval()
    so = o.stats_full_graph(W0, Z0, U0)
    for key in ("objective", "lagrangian", "risk", "primal_res"):
        assert abs(sg[key] - so[key]) <= REL * abs(so[key]), (key, sg[key], so[key])
    for a, b in zip(sg["layer_penalty"], so["layer_penalty"]):
        assert abs(a - b) <= REL * abs(b) + 1e-12 * so["objective"]
    assert sg["status"] == 0
    s.run(1)
    WL1 = s.get_W(L).astype(np.float64)
    ZL1 = g.to_new(s.get_Z(L).astype(np.float64))
    U1 = g.to_new(s.get_U().astype(np.float64))
    TL = g.A @ (Z0[L - 1] @ WL1)
    want = U0 + o.rho * (Z0[L] - TL)
    assert np.abs(U1 - want).max() <= REL * np.abs(want).max()
    rows = np.random.default_rng(index).integers(0, g.N, 2000)
    zref = fista_rows(Z0[L][rows], TL[rows], U0[rows], o.Y[rows], o.labelled[rows], o.rho, o.J, o.risk)
    assert np.abs(ZL1[rows] - zref).max() <= REL * np.abs(zref).max()
    s.close()
