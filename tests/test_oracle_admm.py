"""Pins for the oracle's ADMM part (paper, Section 3 and Appendix A).

Each check ties a piece of the oracle to something other than itself: the augmented
Lagrangian (Eq. 1) written out with dense matrices, finite differences, closed forms,
the inequalities the step parameters must satisfy, and special cases.
"""
import copy
import itertools

import numpy as np
import pytest

from oracle.admm import AdmmOracle, relu
from oracle.graph import OracleGraph

HYPER = dict(nu=0.7, rho=0.3, tau0=1e-3, theta0=1e-3, eta=2.0, max_backtrack=60, fista_iters=10)


def tiny_problem(seed, N=30, M=3, dims=(6, 5, 4, 3), p=0.15, labelled=0.8, hyper=None, risk=0, forward_init=False):
    rng = np.random.default_rng(seed)
    edges = [(u, v) for u, v in itertools.combinations(range(N), 2) if rng.random() < p]
    comm = rng.integers(0, M, size=N).astype(np.int32)
    g = OracleGraph(N, [a for a, _ in edges], [b for _, b in edges], M, comm)
    h = dict(HYPER)
    h.update(hyper or {})
    o = AdmmOracle(g, dims, risk=risk, **h)
    X = rng.standard_normal((N, dims[0]))
    labels = np.where(rng.random(N) < labelled, rng.integers(0, dims[-1], size=N), -1)
    o.set_data(X, labels)
    W0 = [rng.standard_normal((dims[l - 1], dims[l])) * 0.5 for l in range(1, len(dims))]
    o.init(W0)
    if not forward_init:          # a generic point: nothing is stationary, no ReLU argument is near 0
        for l in range(1, o.L + 1):
            o.Z[l] = rng.standard_normal(o.Z[l].shape)
        o.U = rng.standard_normal(o.U.shape)
    return o, rng


def dense_lagrangian(o, W, Z, U):
    """Eq. 1 in its full-graph form, with a dense A~ and explicit loops over layers."""
    A = o.g.A.toarray()
    L = o.L
    zl = Z[L][o.labelled]
    yl = o.Y[o.labelled]
    if o.risk == 0:
        val = float(np.sum(np.log(np.sum(np.exp(zl), axis=1)) - np.sum(yl * zl, axis=1)))
    else:
        val = 0.5 * float(np.sum((zl - yl) ** 2))
    for l in range(1, L):
        val += 0.5 * o.nu * float(np.sum((Z[l] - np.maximum(A @ Z[l - 1] @ W[l], 0.0)) ** 2))
    r = Z[L] - A @ Z[L - 1] @ W[L]
    val += float(np.sum(U * r)) + 0.5 * o.rho * float(np.sum(r * r))
    return val


def messages(o, W):
    p = [o.first_order(l, o.Z[l], W[l + 1]) for l in range(o.L)]
    s = [None] + [o.second_order(l, p[l], o.Z[l + 1], o.U) for l in range(1, o.L)]
    return p, s


# ---------------------------------------------------------------- aggregation and phi
def test_blocked_A_Z_W_equals_brute_force_triple_loop():
    o, rng = tiny_problem(0, N=14, M=3, dims=(3, 4, 2))
    A = o.g.A.toarray()
    Z0, W1 = o.Z[0], o.W[1]
    N, C0, C1 = 14, 3, 4
    want = np.zeros((N, C1))
    for i in range(N):
        for c in range(C1):
            acc = 0.0
            for j in range(N):
                for k in range(C0):
                    acc += A[i, j] * Z0[j, k] * W1[k, c]
            want[i, c] = acc
    got = np.vstack([o.g.aggregate_block(m, Z0) @ W1 for m in range(o.M)])
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-13)


def test_phi_blocked_equals_full_graph_form():
    o, _ = tiny_problem(1)
    A = o.g.A.toarray()
    for l in range(1, o.L):
        want = 0.5 * o.nu * np.sum((o.Z[l] - relu(A @ o.Z[l - 1] @ o.W[l])) ** 2)
        assert o.phi(l, o.W[l], o.Z[l - 1], o.Z[l]) == pytest.approx(want, rel=1e-12)
    L = o.L
    r = o.Z[L] - A @ o.Z[L - 1] @ o.W[L]
    want = np.sum(o.U * r) + 0.5 * o.rho * np.sum(r * r)
    assert o.phi(L, o.W[L], o.Z[L - 1], o.Z[L], o.U) == pytest.approx(want, rel=1e-12)


def test_first_order_messages_sum_to_the_full_aggregation():
    o, _ = tiny_problem(2)
    A = o.g.A.toarray()
    for l in range(o.L):
        p = o.first_order(l, o.Z[l], o.W[l + 1])
        full = A @ o.Z[l] @ o.W[l + 1]
        for m in range(o.M):
            got = sum(p[(r, m)] for r in o.g.nbr_and_self(m))
            np.testing.assert_allclose(got, full[o.g.rows(m)], rtol=0, atol=1e-12)


@pytest.mark.parametrize("l", [1, 2, 3])
def test_grad_phi_matches_central_differences(l):
    o, rng = tiny_problem(3)
    W = o.W[l]
    g = o.grad_phi_W(l, W, o.Z[l - 1], o.Z[l], o.U)
    for _ in range(5):
        d = rng.standard_normal(W.shape)
        h = 1e-6
        fd = (o.phi(l, W + h * d, o.Z[l - 1], o.Z[l], o.U) - o.phi(l, W - h * d, o.Z[l - 1], o.Z[l], o.U)) / (2 * h)
        assert fd == pytest.approx(float(np.sum(g * d)), rel=1e-6, abs=1e-9)


# ---------------------------------------------------------------- psi: message form vs Eq. 1
@pytest.mark.parametrize("seed", [4, 5])
def test_psi_message_form_equals_lagrangian_up_to_a_constant(seed):
    """psi_{l,m}(Z) - psi_{l,m}(Z') must equal L_rho(.., Z_{l,m}=Z, ..) - L_rho(.., Z_{l,m}=Z', ..):
    the second-order messages carry exactly the terms of Eq. 1 that depend on Z_{l,m}."""
    o, rng = tiny_problem(seed)
    p, s = messages(o, o.W)
    for l in range(1, o.L):
        for m in range(o.M):
            rows = o.g.rows(m)
            if rows.stop == rows.start:
                continue
            Za = rng.standard_normal((rows.stop - rows.start, o.dims[l]))
            Zb = rng.standard_normal(Za.shape)
            args = (o.W[l + 1], o.Z[l + 1], o.U, p[l - 1], p[l], s[l])
            d_psi = o.psi(l, m, Za, *args) - o.psi(l, m, Zb, *args)
            vals = []
            for Zx in (Za, Zb):
                Z = [z.copy() for z in o.Z]
                Z[l][rows] = Zx
                vals.append(dense_lagrangian(o, o.W, Z, o.U))
            assert d_psi == pytest.approx(vals[0] - vals[1], rel=1e-10, abs=1e-10)


@pytest.mark.parametrize("seed", [6, 7])
def test_grad_psi_matches_central_differences_and_full_graph_gradient(seed):
    o, rng = tiny_problem(seed)
    p, s = messages(o, o.W)
    A = o.g.A.toarray()
    for l in range(1, o.L):
        # full-graph gradient of Eq. 1 with respect to Z_l at the current point
        Tn = A @ o.Z[l] @ o.W[l + 1]
        if l + 1 < o.L:
            G = o.nu * (relu(Tn) - o.Z[l + 1]) * (Tn > 0)
        else:
            G = -(o.U + o.rho * (o.Z[l + 1] - Tn))
        full = o.nu * (o.Z[l] - relu(A @ o.Z[l - 1] @ o.W[l])) + A.T @ G @ o.W[l + 1].T
        for m in range(o.M):
            rows = o.g.rows(m)
            if rows.stop == rows.start:
                continue
            Z = o.Z[l][rows]
            args = (o.W[l + 1], o.Z[l + 1], o.U, p[l - 1], p[l], s[l])
            g = o.grad_psi(l, m, Z, *args)
            np.testing.assert_allclose(g, full[rows], rtol=1e-10, atol=1e-12)
            for _ in range(3):
                d = rng.standard_normal(Z.shape)
                h = 1e-6
                fd = (o.psi(l, m, Z + h * d, *args) - o.psi(l, m, Z - h * d, *args)) / (2 * h)
                assert fd == pytest.approx(float(np.sum(g * d)), rel=1e-6, abs=1e-9)


# ---------------------------------------------------------------- quadratic models and backtracking
def test_W_step_minimises_the_quadratic_model_and_meets_the_tau_condition():
    o, _ = tiny_problem(8)
    for l in range(1, o.L + 1):
        W = o.W[l]
        phi0 = o.phi(l, W, o.Z[l - 1], o.Z[l], o.U)
        grad = o.grad_phi_W(l, W, o.Z[l - 1], o.Z[l], o.U)
        Wn = o.update_W(l, o.W, o.Z, o.U)
        tau = o.tau[l]
        # gradient of P_l at the new point vanishes:  grad + tau (Wn - W) = 0
        np.testing.assert_allclose(grad + tau * (Wn - W), 0.0, atol=1e-12 * max(1.0, np.abs(grad).max()))
        phin = o.phi(l, Wn, o.Z[l - 1], o.Z[l], o.U)
        model = phi0 + np.sum(grad * (Wn - W)) + 0.5 * tau * np.sum((Wn - W) ** 2)
        assert phin <= model + 1e-12 * abs(model)            # the condition on tau
        assert phin <= phi0                                   # so the subproblem value cannot rise
        assert model == pytest.approx(phi0 - np.sum(grad ** 2) / (2 * tau), rel=1e-12)
        # tau is the first value of the doubling sequence that passes: the one before fails
        if o.trials_W[l] > 1:
            tp = tau / o.eta
            Wp = W - grad / tp
            assert o.phi(l, Wp, o.Z[l - 1], o.Z[l], o.U) > phi0 - np.sum(grad ** 2) / (2 * tp)
            assert tau == pytest.approx(np.float32(HYPER["tau0"]) * o.eta ** (o.trials_W[l] - 1), rel=1e-12)


def test_Z_step_minimises_the_quadratic_model_and_meets_the_theta_condition():
    o, _ = tiny_problem(9)
    p, s = messages(o, o.W)
    searched = 0
    for l in range(1, o.L):
        for m in range(o.M):
            rows = o.g.rows(m)
            if rows.stop == rows.start:
                continue
            Z = o.Z[l][rows]
            args = (o.W[l + 1], o.Z[l + 1], o.U, p[l - 1], p[l], s[l])
            psi0 = o.psi(l, m, Z, *args)
            grad = o.grad_psi(l, m, Z, *args)
            Zn = o.update_Z_hidden(l, m, o.Z, o.W, o.U, p[l - 1], p[l], s[l])
            th = o.theta[l][m]
            np.testing.assert_allclose(grad + th * (Zn - Z), 0.0, atol=1e-12 * max(1.0, np.abs(grad).max()))
            psin = o.psi(l, m, Zn, *args)
            assert psin <= psi0 - np.sum(grad ** 2) / (2 * th) + 1e-12 * abs(psi0)
            if o.trials_Z[l][m] > 1:
                searched += 1
                tp = th / o.eta
                assert o.psi(l, m, Z - grad / tp, *args) > psi0 - np.sum(grad ** 2) / (2 * tp)
    assert searched > 0


def test_backtracking_cap_raises_the_status_bit():
    o, _ = tiny_problem(10, hyper=dict(max_backtrack=1))
    o.iterate(1)
    assert o.status & AdmmOracle.STATUS_BACKTRACK_CAP
    assert max(o.get_steps()[2]) == 2


# ---------------------------------------------------------------- last layer
def test_last_layer_least_squares_has_its_closed_form():
    o, _ = tiny_problem(11, risk=1)
    p, _ = messages(o, o.W)
    A = o.g.A.toarray()
    T = A @ o.Z[o.L - 1] @ o.W[o.L]
    for m in range(o.M):
        rows = o.g.rows(m)
        got = o.update_Z_last(m, o.Z, o.U, p[o.L - 1])
        lab = o.labelled[rows]
        want = (o.Y[rows] + o.rho * T[rows] - o.U[rows]) / (1.0 + o.rho)
        np.testing.assert_allclose(got[lab], want[lab], rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(got[~lab], (T[rows] - o.U[rows] / o.rho)[~lab], rtol=1e-12, atol=1e-12)


def test_last_layer_cross_entropy_fista_approaches_the_newton_solution():
    o, _ = tiny_problem(12)
    p, _ = messages(o, o.W)
    A = o.g.A.toarray()
    T = A @ o.Z[o.L - 1] @ o.W[o.L]
    for m in range(o.M):
        rows = o.g.rows(m)
        lab = o.labelled[rows]
        b = (T[rows] - o.U[rows] / o.rho)
        # per-row Newton on  lse(z) - z_y + rho/2 ||z - b||^2
        want = b.copy()
        for i in np.flatnonzero(lab):
            z = b[i].copy()
            y = o.Y[rows][i]
            for _ in range(100):
                e = np.exp(z - z.max())
                q = e / e.sum()
                grad = q - y + o.rho * (z - b[i])
                H = np.diag(q) - np.outer(q, q) + o.rho * np.eye(z.size)
                z = z - np.linalg.solve(H, grad)
            assert np.max(np.abs(grad)) < 1e-12
            want[i] = z
        errs = []
        for J in (10, 100, 1000):
            got = o.update_Z_last(m, o.Z, o.U, p[o.L - 1], J=J)
            errs.append(np.max(np.abs(got - want)))
            np.testing.assert_allclose(got[~lab], want[~lab], rtol=1e-12, atol=1e-12)   # unlabelled rows: b
        assert errs[2] < 1e-6 and errs[2] < errs[0]
        # J FISTA steps never do worse than the start on the subproblem's own objective
        start = o.psi_last(m, o.Z[o.L][rows], o.U, p[o.L - 1])
        assert o.psi_last(m, o.update_Z_last(m, o.Z, o.U, p[o.L - 1]), o.U, p[o.L - 1]) < start


def test_psi_last_equals_lagrangian_up_to_a_constant():
    o, rng = tiny_problem(13)
    p, _ = messages(o, o.W)
    for m in range(o.M):
        rows = o.g.rows(m)
        Za, Zb = (rng.standard_normal((rows.stop - rows.start, o.dims[-1])) for _ in range(2))
        vals = []
        for Zx in (Za, Zb):
            Z = [z.copy() for z in o.Z]
            Z[o.L][rows] = Zx
            vals.append(dense_lagrangian(o, o.W, Z, o.U))
        d = o.psi_last(m, Za, o.U, p[o.L - 1]) - o.psi_last(m, Zb, o.U, p[o.L - 1])
        assert d == pytest.approx(vals[0] - vals[1], rel=1e-10, abs=1e-10)


# ---------------------------------------------------------------- whole sweep
def test_forward_pass_start_has_zero_penalties_and_zero_residual():
    o, _ = tiny_problem(14, forward_init=True)
    st = o.stats()
    assert st["primal_res"] == 0.0 and all(v == 0.0 for v in st["layer_penalty"])
    assert st["objective"] == st["risk"] == st["lagrangian"]
    for l in range(1, o.L + 1):
        assert np.all(o.grad_phi_W(l, o.W[l], o.Z[l - 1], o.Z[l], o.U) == 0.0)


def test_sweep_is_jacobi_dual_step_and_readout_are_consistent():
    o, _ = tiny_problem(15)
    A = o.g.A.toarray()
    W0, Z0, U0 = copy.deepcopy(o.W), copy.deepcopy(o.Z), o.U.copy()
    o.iterate(1)
    # W^{k+1} depends on (W^k, Z^k, U^k) only: recompute each layer alone from the saved iterate
    o2, _ = tiny_problem(15)
    for l in range(1, o.L + 1):
        np.testing.assert_array_equal(o2.update_W(l, W0, Z0, U0), o.W[l])
    # dual step as printed (Eq. 2): U^{k+1} - U^k = rho (Z_L^k - A~ Z_{L-1}^k W_L^{k+1})
    r = Z0[o.L] - A @ Z0[o.L - 1] @ o.W[o.L]
    np.testing.assert_allclose(o.U - U0, o.rho * r, rtol=1e-10, atol=1e-12)
    assert np.linalg.norm(o.U - U0) == pytest.approx(o.rho * np.linalg.norm(r), rel=1e-10)
    # readout against Eq. 1 written densely
    st = o.stats()
    assert st["lagrangian"] == pytest.approx(dense_lagrangian(o, o.W, o.Z, o.U), rel=1e-11)
    assert st["primal_res"] == pytest.approx(np.linalg.norm(o.Z[o.L] - A @ o.Z[o.L - 1] @ o.W[o.L]), rel=1e-11)
    assert st["dual_res"] == pytest.approx(
        o.rho * np.linalg.norm(A @ o.Z[o.L - 1] @ o.W[o.L] - A @ Z0[o.L - 1] @ W0[o.L]), rel=1e-10)
    # every Z_{l,m}^{k+1} lowers L_rho(W^{k+1}, Z^k with that block replaced, U^k)
    for l in range(1, o.L + 1):
        for m in range(o.M):
            rows = o.g.rows(m)
            Z = [z.copy() for z in Z0]
            Z[l][rows] = o.Z[l][rows]
            assert dense_lagrangian(o, o.W, Z, U0) <= dense_lagrangian(o, o.W, Z0, U0) + 1e-10


def test_full_graph_readout_equals_blocked_readout():
    o, _ = tiny_problem(19)
    o.iterate(2)
    a, b = o.stats(), o.stats_full_graph()
    for key in ("objective", "lagrangian", "risk", "primal_res"):
        assert b[key] == pytest.approx(a[key], rel=1e-12)
    for l in range(1, o.L + 1):
        assert o.phi_full_graph(l, o.W[l], o.Z[l - 1], o.Z[l], o.U) == pytest.approx(
            o.phi(l, o.W[l], o.Z[l - 1], o.Z[l], o.U), rel=1e-12)


def test_predict_is_the_forward_pass_with_a_dense_adjacency():
    o, _ = tiny_problem(20, forward_init=True)
    o.iterate(3)
    A = o.g.A.toarray()
    Z = o.Z[0]
    for l in range(1, o.L + 1):
        T = A @ Z @ o.W[l]
        Z = np.maximum(T, 0.0) if l < o.L else T
    pred, logits, acc = o.predict()
    np.testing.assert_allclose(o.g.to_new(logits), Z, rtol=1e-12, atol=1e-13)
    assert np.array_equal(o.g.to_new(pred), np.argmax(Z, axis=1))
    lab = o.labelled
    assert acc == pytest.approx(np.mean(np.argmax(Z, axis=1)[lab] == o.labels[lab]))
    # at the forward-pass start the last layer's state is exactly these logits
    o2, _ = tiny_problem(20, forward_init=True)
    np.testing.assert_allclose(o2.predict()[1], o2.get_Z(o2.L), rtol=1e-12, atol=1e-13)


def test_dual_form_1_is_dual_ascent_on_the_new_iterates():
    o, _ = tiny_problem(21, hyper=dict(dual_form=1))
    o0, _ = tiny_problem(21)
    A = o.g.A.toarray()
    U0 = o.U.copy()
    o.iterate(1)
    o0.iterate(1)
    r_new = o.Z[o.L] - A @ o.Z[o.L - 1] @ o.W[o.L]
    np.testing.assert_allclose(o.U - U0, o.rho * r_new, rtol=1e-10, atol=1e-12)
    assert o.stats()["primal_res"] == pytest.approx(np.linalg.norm(o.U - U0) / o.rho, rel=1e-10)
    # W and Z of the first iteration do not depend on the form of the dual step; U does
    for l in range(1, o.L + 1):
        np.testing.assert_array_equal(o.W[l], o0.W[l])
        np.testing.assert_array_equal(o.Z[l], o0.Z[l])
    assert np.abs(o.U - o0.U).max() > 1e-3


def test_disconnected_communities_decouple_in_the_Z_update():
    """Without inter-community edges N_m is empty, no s-terms exist, and Z_{l,m}^{k+1} equals what a
    one-community problem on the subgraph of V_m alone produces from the same W^{k+1}."""
    rng = np.random.default_rng(16)
    N, M, dims = 24, 3, (4, 5, 3)
    comm = np.repeat(np.arange(M), N // M).astype(np.int32)
    edges = [(u, v) for u, v in itertools.combinations(range(N), 2) if comm[u] == comm[v] and rng.random() < 0.3]
    g = OracleGraph(N, [a for a, _ in edges], [b for _, b in edges], M, comm)
    assert not g.neighbour.any()
    X = rng.standard_normal((N, dims[0]))
    labels = rng.integers(0, dims[-1], size=N)
    W0 = [rng.standard_normal((dims[l - 1], dims[l])) for l in range(1, 3)]
    big = AdmmOracle(g, dims, **HYPER)
    big.set_data(X, labels)
    big.init(W0)
    Zr = [None] + [rng.standard_normal(big.Z[l].shape) for l in (1, 2)]
    Ur = rng.standard_normal(big.U.shape)
    big.Z[1:] = [z.copy() for z in Zr[1:]]
    big.U = Ur.copy()
    p = [big.first_order(l, big.Z[l], big.W[l + 1]) for l in range(2)]
    s = [None, big.second_order(1, p[1], big.Z[2], big.U)]
    for m in range(M):
        idx = np.flatnonzero(comm == m)
        loc = {int(o_): i for i, o_ in enumerate(idx)}
        sub_edges = [(loc[u], loc[v]) for u, v in edges if comm[u] == m]
        gs = OracleGraph(len(idx), [a for a, _ in sub_edges], [b for _, b in sub_edges], 1, None)
        # degrees inside an isolated community are the same as in the union graph
        small = AdmmOracle(gs, dims, **HYPER)
        small.set_data(X[idx], labels[idx])
        small.init(W0)
        small.Z[1], small.Z[2], small.U = Zr[1][idx], Zr[2][idx], Ur[idx]
        ps = [small.first_order(l, small.Z[l], small.W[l + 1]) for l in range(2)]
        ss = [None, small.second_order(1, ps[1], small.Z[2], small.U)]
        want = small.update_Z_hidden(1, 0, small.Z, small.W, small.U, ps[0], ps[1], ss[1])
        got = big.update_Z_hidden(1, m, big.Z, big.W, big.U, p[0], p[1], s[1])
        np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)


def test_relabelling_nodes_and_communities_leaves_the_iterates_unchanged():
    rng = np.random.default_rng(17)
    N, M, dims = 40, 4, (5, 6, 4, 3)
    edges = [(u, v) for u, v in itertools.combinations(range(N), 2) if rng.random() < 0.1]
    comm = rng.integers(0, M, size=N).astype(np.int32)
    X = rng.standard_normal((N, dims[0]))
    labels = rng.integers(0, dims[-1], size=N)
    W0 = [rng.standard_normal((dims[l - 1], dims[l])) * 0.5 for l in range(1, len(dims))]
    hyper = dict(HYPER, nu=1e-2, rho=1e-2)

    def run(node_map, comm_map):
        comm2 = np.empty(N, dtype=np.int32)
        comm2[node_map] = comm_map[comm]
        X2 = np.empty_like(X)
        X2[node_map] = X
        lab2 = np.empty_like(labels)
        lab2[node_map] = labels
        g = OracleGraph(N, [node_map[a] for a, _ in edges], [node_map[b] for _, b in edges], M, comm2)
        o = AdmmOracle(g, dims, **hyper)
        o.set_data(X2, lab2)
        o.init(W0)
        o.iterate(4)
        return o, [o.get_Z(l)[node_map] for l in range(1, o.L + 1)]

    oa, Za = run(np.arange(N), np.arange(M))
    ob, Zb = run(rng.permutation(N), rng.permutation(M))
    for l in range(1, oa.L + 1):
        np.testing.assert_allclose(ob.W[l], oa.W[l], rtol=1e-9, atol=1e-11)
        np.testing.assert_allclose(Zb[l - 1], Za[l - 1], rtol=1e-9, atol=1e-11)
    assert ob.stats()["objective"] == pytest.approx(oa.stats()["objective"], rel=1e-10)


def test_empty_graph_reduces_to_a_plain_multilayer_perceptron_penalty():
    rng = np.random.default_rng(18)
    N, dims = 12, (3, 4, 2)
    g = OracleGraph(N, [], [], 2, None)
    o = AdmmOracle(g, dims, **HYPER)
    X = rng.standard_normal((N, 3))
    o.set_data(X, rng.integers(0, 2, size=N))
    o.init([rng.standard_normal((3, 4)), rng.standard_normal((4, 2))])
    o.Z[1] = rng.standard_normal((N, 4))
    assert o.phi(1, o.W[1], o.Z[0], o.Z[1]) == pytest.approx(
        0.5 * o.nu * np.sum((o.Z[1] - relu(o.Z[0] @ o.W[1])) ** 2), rel=1e-13)


# ---------------------------------------------------------------- serial baseline: layer by layer (Section 4.1)
def test_layer_by_layer_pass_descends_the_lagrangian_at_every_W_and_hidden_Z_block():
    # one community: every block update is then an exact Gauss-Seidel step on Eq. 1, and backtracking on a
    # majorising model cannot increase it (the FISTA block carries momentum and is not checked)
    o, _ = tiny_problem(31, M=1, hyper=dict(schedule=1))
    for _ in range(3):
        before = dense_lagrangian(o, o.W, o.Z, o.U)
        o.block_trace = []
        o.iterate(1)
        assert [(n, l) for n, l, _ in o.block_trace] == [("W", 1), ("Z", 1), ("W", 2), ("Z", 2), ("W", 3), ("Z", 3)]
        prev = before
        for name, l, val in o.block_trace:
            if not (name == "Z" and l == o.L):
                assert val <= prev + 1e-10 * abs(prev), (name, l, val, prev)
            prev = val
        assert o.block_trace[-2][2] < before - 1e-6 * abs(before)      # and the pass does move
    assert o.status == 0


def test_layer_by_layer_feeds_each_block_the_newest_values():
    o, _ = tiny_problem(32, hyper=dict(schedule=1))
    j, _ = tiny_problem(32)                          # Algorithm 1 from the same point
    A = o.g.A.toarray()
    W_old = [None] + [w.copy() for w in o.W[1:]]
    Z_old = [z.copy() for z in o.Z]
    U_old = o.U.copy()
    o.iterate(1)
    j.iterate(1)
    # the first block sees the same inputs in both schedules
    np.testing.assert_array_equal(o.W[1], j.W[1])
    # W_2 is a gradient step of phi_2 taken at Z_1^{k+1}: rebuild it densely with the accepted tau_2
    H = A @ o.Z[1]
    T = H @ W_old[2]
    G = o.nu * (np.maximum(T, 0.0) - Z_old[2]) * (T > 0)
    np.testing.assert_allclose(o.W[2], W_old[2] - (H.T @ G) / o.tau[2], rtol=1e-11, atol=1e-13)
    assert np.abs(o.W[2] - j.W[2]).max() > 1e-6       # Algorithm 1 took it at Z_1^k
    # Z_2 saw W_2^{k+1}, Z_1^{k+1} (through T_2) and the old W_3, Z_3
    for m in range(o.M):
        rows = o.g.rows(m)
        def psi_dense(Zm):
            Z2 = Z_old[2].copy()
            Z2[rows] = Zm
            own = 0.5 * o.nu * np.sum((Zm - np.maximum(A[rows] @ o.Z[1] @ o.W[2], 0.0)) ** 2)
            r = Z_old[3] - A @ Z2 @ W_old[3]          # rows not adjacent to V_m only add a constant
            return own + np.sum(U_old * r) + 0.5 * o.rho * np.sum(r * r)
        eps = 1e-6
        rng = np.random.default_rng(5 + m)
        D = rng.standard_normal(Z_old[2][rows].shape)
        g_fd = (psi_dense(Z_old[2][rows] + eps * D) - psi_dense(Z_old[2][rows] - eps * D)) / (2 * eps)
        step = (Z_old[2][rows] - o.Z[2][rows]) * o.theta[2][m]          # = grad psi at the old block
        assert np.sum(step * D) == pytest.approx(g_fd, rel=1e-5, abs=1e-8)
    # dual step of form 0: Z_L^k and the T_L the last-layer update saw
    np.testing.assert_allclose(o.U - U_old, o.rho * (Z_old[3] - A @ o.Z[2] @ o.W[3]), rtol=1e-10, atol=1e-12)


def test_layer_by_layer_with_dual_form_1_uses_the_new_last_layer():
    o, _ = tiny_problem(33, hyper=dict(schedule=1, dual_form=1))
    A = o.g.A.toarray()
    U_old = o.U.copy()
    o.iterate(1)
    np.testing.assert_allclose(o.U - U_old, o.rho * (o.Z[3] - A @ o.Z[2] @ o.W[3]), rtol=1e-10, atol=1e-12)


# ---------------------------------------------------------------- step parameters that may shrink again
def test_step_policy_1_starts_a_search_one_notch_lower_and_still_meets_the_conditions():
    o, _ = tiny_problem(41, hyper=dict(step_policy=1))
    m, _ = tiny_problem(41)                                       # monotone policy from the same point
    for _ in range(6):
        o.iterate(1)
        m.iterate(1)
    assert o.status == 0
    # the first search of a run starts at tau0 / eta, so an accepted value below tau0 * eta^j of the monotone run shows up
    taus_o, taus_m = np.array(o.tau[1:]), np.array(m.tau[1:])
    assert np.all(np.log2(taus_o / o.tau[1]) % 1 == 0)            # still powers of eta apart
    assert np.any(taus_o < taus_m)                                # some parameter ended lower than the monotone one
    # an accepted tau satisfies the model condition at the point it was taken from: redo the last W step densely
    A = o.g.A.toarray()
    snap = o.snapshot()
    W_old, Z_old = [None] + [w.copy() for w in o.W[1:]], [z.copy() for z in o.Z]
    tau_before = list(o.tau)
    o.iterate(1)
    l = 1
    H = A @ Z_old[0]
    T = H @ W_old[1]
    G = o.nu * (np.maximum(T, 0.0) - Z_old[1]) * (T > 0)
    grad = H.T @ G
    tau = o.tau[1]
    assert tau >= tau_before[1] / o.eta * (1 - 1e-12)             # never below the first candidate
    Wn = W_old[1] - grad / tau
    phi = lambda W: 0.5 * o.nu * np.sum((Z_old[1] - np.maximum(H @ W, 0.0)) ** 2)
    assert phi(Wn) <= phi(W_old[1]) - np.sum(grad * grad) / (2 * tau) + 1e-12 * abs(phi(W_old[1]))
    np.testing.assert_allclose(o.W[1], Wn, rtol=1e-11, atol=1e-13)
    if tau > tau_before[1] / o.eta * (1 + 1e-12):                 # then the candidate before it failed the condition
        Wp = W_old[1] - grad / (tau / o.eta)
        assert phi(Wp) > phi(W_old[1]) - np.sum(grad * grad) / (2 * tau / o.eta)
    o.restore(snap)


# ---------------------------------------------------------------- a step below resolution is not taken
def _floor_case(seed):
    o, _ = tiny_problem(seed)
    o.iterate(2)                      # a generic state with step parameters that have been searched
    return o


def test_step_floor_of_the_W_update_has_its_boundary_where_the_reading_puts_it():
    """Reading: if the first candidate would move W_l by less than 1e-12 of its norm, ||grad||^2 <= (1e-12 tau)^2 ||W||^2,
    the block and tau_l stay and no trial is counted.  tau is placed just above and just below ||grad|| / (1e-12 ||W||)
    for a gradient that is far from zero."""
    o = _floor_case(21)
    for l in range(1, o.L + 1):
        W = o.W[l].copy()
        grad = o.grad_phi_W(l, W, o.Z[l - 1], o.Z[l], o.U)
        gn, wn = np.sqrt(np.sum(grad ** 2)), np.sqrt(np.sum(W ** 2))
        assert gn > 1e-6 * wn                                  # nothing like a zero gradient
        edge = gn / (AdmmOracle.STEP_FLOOR * wn)               # tau at which the first step has relative size 1e-12
        # at or beyond the edge: nothing moves, nothing is counted, tau is kept
        for tau in (edge * (1 + 1e-9), edge * 4.0):
            o.tau[l], o.trials_W[l] = tau, -7
            Wn = o.update_W(l, o.W, o.Z, o.U)
            assert np.array_equal(Wn, W) and Wn is not o.W[l]
            assert o.tau[l] == tau and o.trials_W[l] == 0
        # just inside: the step is taken, with at least one trial, and it is the model's minimiser for the tau it ends with
        o.tau[l] = edge * (1 - 1e-6)
        Wn = o.update_W(l, o.W, o.Z, o.U)
        assert o.trials_W[l] >= 1 and o.tau[l] >= edge * (1 - 1e-6)
        assert not np.array_equal(Wn, W)
        np.testing.assert_allclose(Wn, W - grad / o.tau[l], rtol=0, atol=0)
        moved = np.sqrt(np.sum((Wn - W) ** 2)) / wn
        assert 0 < moved <= 1.01e-12


def test_step_floor_of_the_Z_update_has_its_boundary_where_the_reading_puts_it():
    o = _floor_case(22)
    p, s = messages(o, o.W)
    checked = 0
    for l in range(1, o.L):
        for m in range(o.M):
            rows = o.g.rows(m)
            if rows.stop == rows.start:
                continue
            Z = o.Z[l][rows].copy()
            args = (o.W[l + 1], o.Z[l + 1], o.U, p[l - 1], p[l], s[l])
            grad = o.grad_psi(l, m, Z, *args)
            gn, zn = np.sqrt(np.sum(grad ** 2)), np.sqrt(np.sum(Z ** 2))
            assert gn > 1e-6 * zn
            edge = gn / (AdmmOracle.STEP_FLOOR * zn)
            o.theta[l][m], o.trials_Z[l][m] = edge * (1 + 1e-9), -7
            Zn = o.update_Z_hidden(l, m, o.Z, o.W, o.U, p[l - 1], p[l], s[l])
            assert np.array_equal(Zn, Z) and o.theta[l][m] == edge * (1 + 1e-9) and o.trials_Z[l][m] == 0
            o.theta[l][m] = edge * (1 - 1e-6)
            Zn = o.update_Z_hidden(l, m, o.Z, o.W, o.U, p[l - 1], p[l], s[l])
            assert o.trials_Z[l][m] >= 1 and not np.array_equal(Zn, Z)
            np.testing.assert_allclose(Zn, Z - grad / o.theta[l][m], rtol=0, atol=0)
            checked += 1
    assert checked >= 2


def test_step_floor_uses_the_first_candidate_of_the_search_under_step_policy_1():
    """With step_policy 1 the first candidate is tau / eta, and the floor is taken at that value."""
    o, _ = tiny_problem(23, hyper=dict(step_policy=1))
    o.iterate(2)
    l = 1
    W = o.W[l].copy()
    grad = o.grad_phi_W(l, W, o.Z[l - 1], o.Z[l], o.U)
    edge = np.sqrt(np.sum(grad ** 2)) / (AdmmOracle.STEP_FLOOR * np.sqrt(np.sum(W ** 2)))
    o.tau[l] = edge * o.eta * (1 + 1e-9)           # first candidate just beyond the edge
    assert np.array_equal(o.update_W(l, o.W, o.Z, o.U), W) and o.trials_W[l] == 0
    o.tau[l] = edge * o.eta * (1 - 1e-6)
    assert not np.array_equal(o.update_W(l, o.W, o.Z, o.U), W) and o.trials_W[l] >= 1


# ---------------------------------------------------------------- the ReLU-tie hook of the parity tests
def test_relu_tie_hook_flips_only_named_entries_inside_the_band_and_is_off_by_default():
    import oracle.admm as oa
    hook = oa.RELU_TIES
    o, rng = tiny_problem(24)
    l = 1
    # plant a pre-activation that is zero up to 1e-9 of the block's rms: solve for one entry of Z_0... simpler, shift
    # one column of W_1 so that T_1[i, j] of community m's block lands at +1e-9 rms
    m = max(range(o.M), key=lambda q: o.g.rows(q).stop - o.g.rows(q).start)
    rows = o.g.rows(m)
    H = o.g.aggregate_block(m, o.Z[0])
    T = H @ o.W[l]
    i, j = 1, 2
    rms = np.sqrt(np.mean(T * T))
    k = int(np.argmax(np.abs(H[i])))
    o.W[l][k, j] += (1e-9 * rms - T[i, j]) / H[i, k]
    T = H @ o.W[l]
    assert 0 < T[i, j] < 1e-8 * rms
    key = ("W", l, rows.start + i, j)
    try:
        g_plain = o.grad_phi_W(l, o.W[l], o.Z[0], o.Z[l])
        assert hook.found == {} and hook.flipped == {}                      # off by default: nothing recorded
        hook.band = 4e-6
        g_probe = o.grad_phi_W(l, o.W[l], o.Z[0], o.Z[l])
        assert np.array_equal(g_probe, g_plain)                             # recording changes nothing
        assert list(hook.found) == [key]                                    # and finds exactly the planted entry
        far = ("W", l, rows.start, 0)
        hook.flips = {key, far}                                             # an entry outside the band cannot be flipped
        g_flip = o.grad_phi_W(l, o.W[l], o.Z[0], o.Z[l])
        assert set(hook.flipped) == {key}
        # the flipped derivative is 0 instead of 1 at that entry: the gradient loses exactly H_i^T G_ij
        Gij = o.nu * (max(T[i, j], 0.0) - o.Z[l][rows][i, j])
        expect = g_plain.copy()
        expect[:, j] -= H[i] * Gij
        np.testing.assert_allclose(g_flip, expect, rtol=1e-12, atol=1e-15)
    finally:
        hook.reset()
    assert np.array_equal(o.grad_phi_W(l, o.W[l], o.Z[0], o.Z[l]), g_plain)


# ---------------------------------------------------------------- last layer by FISTA with backtracking (fista_mode 1)
def test_fista_backtracking_least_squares_finds_the_curvature_and_the_closed_form():
    """For the least-squares risk the block objective is a quadratic with Hessian (1 + rho) I: the condition
    F(y - g/L) <= F(y) - ||g||^2 / (2L) holds exactly when L >= 1 + rho, so the search must stop at the first
    rho eta^i that reaches 1 + rho, in the first step, and the iterates must tend to the closed-form minimiser."""
    o, _ = tiny_problem(31, risk=1, hyper=dict(fista_mode=1, rho=0.3))
    p, _ = messages(o, o.W)
    A = o.g.A.toarray()
    T = A @ o.Z[o.L - 1] @ o.W[o.L]
    i = 0
    while o.rho * o.eta ** i < 1.0 + o.rho:
        i += 1
    for m in range(o.M):
        rows = o.g.rows(m)
        lab = o.labelled[rows]
        if not lab.any():
            continue
        got1 = o.update_Z_last(m, o.Z, o.U, p[o.L - 1], J=1)
        assert o.fista_L[m] == pytest.approx(o.rho * o.eta ** i, rel=1e-12) and o.fista_trials[m] == i + 1
        # the first step from y = Z_L is the plain gradient step of length 1/L
        z0 = o.Z[o.L][rows]
        g = o.U[rows] + o.rho * (z0 - T[rows]) + (z0 - o.Y[rows])
        np.testing.assert_allclose(got1[lab], (z0 - g / o.fista_L[m])[lab], rtol=1e-12, atol=1e-12)
        want = (o.Y[rows] + o.rho * T[rows] - o.U[rows]) / (1.0 + o.rho)
        got12 = o.update_Z_last(m, o.Z, o.U, p[o.L - 1], J=12)
        assert o.fista_trials[m] == 12 + i                        # no growth after the first step
        got = o.update_Z_last(m, o.Z, o.U, p[o.L - 1], J=40)
        np.testing.assert_allclose(got[lab], want[lab], rtol=0, atol=1e-6)
        assert np.abs(got[lab] - want[lab]).max() < np.abs(got12[lab] - want[lab]).max()
        np.testing.assert_allclose(got[~lab], (T[rows] - o.U[rows] / o.rho)[~lab], rtol=1e-12, atol=1e-12)


def test_fista_backtracking_meets_its_condition_with_the_first_L_that_does():
    """Cross-entropy, every row labelled, one step: with the accepted L the new block satisfies
    psi(x) <= psi(y) - ||grad||^2 / (2L) on the subproblem's objective (psi_last, pinned to Eq. 1 above), with
    L / eta it does not, and L is rho times a power of eta."""
    o, _ = tiny_problem(32, labelled=1.0, hyper=dict(fista_mode=1, rho=0.05))
    p, _ = messages(o, o.W)
    A = o.g.A.toarray()
    T = A @ o.Z[o.L - 1] @ o.W[o.L]
    searched = 0
    for m in range(o.M):
        rows = o.g.rows(m)
        if rows.stop == rows.start:
            continue
        z0 = o.Z[o.L][rows]
        e = np.exp(z0 - z0.max(axis=1, keepdims=True))
        g = e / e.sum(axis=1, keepdims=True) - o.Y[rows] + o.U[rows] + o.rho * (z0 - T[rows])
        x = o.update_Z_last(m, o.Z, o.U, p[o.L - 1], J=1)
        L = o.fista_L[m]
        k = np.log(L / o.rho) / np.log(o.eta)
        assert abs(k - round(k)) < 1e-9 and round(k) == o.fista_trials[m] - 1
        np.testing.assert_allclose(x, z0 - g / L, rtol=1e-12, atol=1e-12)
        psi = lambda z: o.psi_last(m, z, o.U, p[o.L - 1])
        gg = float(np.sum(g * g))
        assert psi(x) <= psi(z0) - gg / (2 * L) + 1e-12 * abs(psi(z0))
        if o.fista_trials[m] > 1:
            searched += 1
            Lp = L / o.eta
            assert psi(z0 - g / Lp) > psi(z0) - gg / (2 * Lp)
    assert searched > 0


def test_fista_backtracking_approaches_the_newton_solution_and_stays_below_twice_the_curvature_bound():
    o, _ = tiny_problem(33, hyper=dict(fista_mode=1))
    o0, _ = tiny_problem(33, hyper=dict(fista_mode=0))
    p, _ = messages(o, o.W)
    A = o.g.A.toarray()
    T = A @ o.Z[o.L - 1] @ o.W[o.L]
    for m in range(o.M):
        rows = o.g.rows(m)
        lab = o.labelled[rows]
        if not lab.any():
            continue
        b = T[rows] - o.U[rows] / o.rho
        want = b.copy()
        for i in np.flatnonzero(lab):
            z = b[i].copy()
            y = o.Y[rows][i]
            for _ in range(200):
                e = np.exp(z - z.max())
                q = e / e.sum()
                grad = q - y + o.rho * (z - b[i])
                z = z - np.linalg.solve(np.diag(q) - np.outer(q, q) + o.rho * np.eye(z.size), grad)
            assert np.max(np.abs(grad)) < 1e-12
            want[i] = z
        got = o.update_Z_last(m, o.Z, o.U, p[o.L - 1], J=1000)
        np.testing.assert_allclose(got, want, rtol=0, atol=1e-6)
        assert o.fista_L[m] <= o.eta * (o.rho + 0.5)             # never beyond the first candidate above the bound
        # both modes head for the same point
        np.testing.assert_allclose(o0.update_Z_last(m, o0.Z, o0.U, p[o.L - 1], J=1000), want, rtol=0, atol=1e-6)


def test_fista_backtracking_cap_raises_the_status_bit_and_the_sweep_stays_consistent():
    o, _ = tiny_problem(34, hyper=dict(fista_mode=1, rho=1e-3, max_backtrack=2))
    o.iterate(1)
    assert o.status & AdmmOracle.STATUS_BACKTRACK_CAP
    o, _ = tiny_problem(35, hyper=dict(fista_mode=1))
    A = o.g.A.toarray()
    Z0, U0 = copy.deepcopy(o.Z), o.U.copy()
    o.iterate(1)
    TL = A @ Z0[o.L - 1] @ o.W[o.L]
    np.testing.assert_allclose(o.U, U0 + o.rho * (Z0[o.L] - TL), rtol=1e-12, atol=1e-12)     # Eq. 2 is untouched by the mode
