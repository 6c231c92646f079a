"""GPU parity of the whole ADMM sweep against the CPU oracle, iteration by iteration, on the same seeded
inputs (tolerance 1e-4 relative on W, Z, U and the objective; step-size trajectories identical)."""
import copy

import numpy as np
import pytest

from oracle.admm import make_oracle
from paper_2112_09335_amd import synth
from parity import compare_iterate, expected_ties, record_case, say, step_with_relu_ties

pytestmark = pytest.mark.gpu


def run_case(w, iters, tag, max_ties=None, tune=None):
    """Per-iteration parity of one workload.  A hidden pre-activation within fp32 rounding of zero (a ReLU tie, see
    step_with_relu_ties) is accepted only entry by entry, and in at most max_ties iterations of the case: the number
    of tied entries expected for its size and length (parity.expected_ties) rounded up, at least one."""
    max_ties = max(1, int(np.ceil(expected_ties(w.N, w.dims, iters)))) if max_ties is None else max_ties
    from paper_2112_09335_amd import binding
    say(f"[{tag}] N={w.N} M={w.M} dims={w.dims} E={w.E} iters={iters}")
    solver = binding.Solver.from_workload(w, 0)
    for key, value in (tune or {}).items():
        solver.tune(key, value)
    orc = make_oracle(w)
    ties, worst, done = [], 0.0, 0
    try:
        worst = compare_iterate(solver, orc, f"{tag} it0")
        for k in range(1, iters + 1):
            err, flipped = step_with_relu_ties(solver, orc, f"{tag} it{k}")
            worst = max(worst, err)
            if flipped:
                ties.append(dict(iter=k, entries=flipped))
            done = k
            say(f"[{tag}] it{k} ok, worst rel err so far {worst:.2e}")
        assert len(ties) <= max_ties, f"{len(ties)} iterations with ReLU ties in {iters} iterations"
    finally:
        solver.close()
        record_case(case=tag, N=int(w.N), dims=list(w.dims), iters=iters, iters_done=done, worst=worst, ties=ties,
                    max_ties=max_ties, expected_ties=expected_ties(w.N, w.dims, iters),
                    ok=bool(done == iters and len(ties) <= max_ties))
    return worst


def test_config1_tiny_sbm_all_iterations():
    w = synth.config(1)
    run_case(w, w.iters, "config1")


def test_config2_mid_sbm_scaled():
    w = synth.config(2, 0.1)             # N = 2000, 500 -> 128 -> 3
    run_case(w, 12, "config2/10")


def test_config3_three_layers_scaled():
    w = synth.config(3, 0.01)            # N = 2000, 32 communities, 128 -> 256 -> 256 -> 10
    run_case(w, 8, "config3/100")


def test_config4_powerlaw_scaled():
    w = synth.config(4, 0.002)           # N = 4000, 64 communities, hubs, 128 -> 256 -> 16
    run_case(w, 8, "config4/500")


def test_config5_deep_scaled():
    w = synth.config(5, 0.002, M=4)      # N = 1000, 8 layers of 512
    run_case(w, 4, "config5/500")


def test_unlabelled_nodes_least_squares_risk_one_community_and_ragged_sizes():
    w = synth.make_workload("ragged", 11, 1237, 5, [37, 50, 9, 6], 6, 6, graph="sbm", features="gaussian",
                            avg_degree=6, frac_intra=0.7, labelled_fraction=0.4)
    w.comm = np.where(w.comm == 3, 4, w.comm).astype(np.int32)      # community 3 is empty
    run_case(w, 6, "ragged-ce")
    w2 = copy.deepcopy(w)
    w2.hyper["risk"] = 1
    run_case(w2, 4, "ragged-lsq")
    w3 = synth.make_workload("single", 12, 600, 1, [20, 33, 4], 4, 5, graph="sbm", features="gaussian",
                             avg_degree=8, frac_intra=1.0)
    run_case(w3, 5, "one-community")
    w4 = synth.make_workload("noedges", 13, 300, 3, [10, 12, 3], 3, 3, graph="empty", features="gaussian")
    run_case(w4, 3, "empty-graph")


def test_backtracking_cap_status_and_resume_are_consistent():
    from paper_2112_09335_amd import binding
    w = synth.config(1, 0.5)
    w.hyper["max_backtrack"] = 2
    run_case(w, 3, "cap")                # both sides must raise the same status bit
    # resume: 4 iterations == 2 iterations, state out and in again, 2 more (bit for bit on the GPU side)
    # (the first layer's pre-activation is normally carried across iterations; a resumed run has to form
    # it anew, so for a bit-for-bit comparison every run forms it in every iteration)
    w = synth.config(1, 0.5)
    a = binding.Solver.from_workload(w, 0)
    a.tune("t1_refresh", 0)
    a.run(4)
    b = binding.Solver.from_workload(w, 0)
    b.tune("t1_refresh", 0)
    b.run(2)
    tau, theta, _, _ = b.get_steps()
    W = [b.get_W(l) for l in range(1, w.L + 1)]
    Z = [b.get_Z(l) for l in range(1, w.L + 1)]
    U = b.get_U()
    c = binding.Solver.from_workload(w, 0)
    c.tune("t1_refresh", 0)
    c.set_state(W=W, Z=Z, U=U, tau=tau, theta=theta)
    c.run(2)
    for l in range(1, w.L + 1):
        assert np.array_equal(a.get_W(l), c.get_W(l))
        assert np.array_equal(a.get_Z(l), c.get_Z(l))
    assert np.array_equal(a.get_U(), c.get_U())
    # and the run itself is reproducible bit for bit
    d = binding.Solver.from_workload(w, 0)
    d.tune("t1_refresh", 0)
    d.run(4)
    assert np.array_equal(a.get_Z(1), d.get_Z(1)) and a.eval()["objective"] == d.eval()["objective"]
    # carrying the first layer's pre-activation changes the iterates only by rounding
    e = binding.Solver.from_workload(w, 0)
    e.run(4)
    assert np.abs(e.get_Z(1) - a.get_Z(1)).max() <= 1e-5 * np.abs(a.get_Z(1)).max()
    e.close()
    for s in (a, b, c, d):
        s.close()


def test_graph_replay_equals_plain_launches_bit_for_bit():
    """cadmm_run replays a captured HIP graph; with readouts (eager kernels, synchronisations) between the
    replays every iterate must equal the one from plain launches exactly."""
    from paper_2112_09335_amd import binding
    w = synth.config(2, 0.1)
    a = binding.Solver.from_workload(w, 0)
    b = binding.Solver.from_workload(w, 0)
    b.tune("use_graph", 0)
    for k in range(6):
        a.run(1 if k % 2 == 0 else 2)
        b.run(1 if k % 2 == 0 else 2)
        sa, sb = a.eval(), b.eval()
        assert sa == sb, (k, sa, sb)
        for l in range(1, w.L + 1):
            assert np.array_equal(a.get_W(l), b.get_W(l)), (k, l)
            assert np.array_equal(a.get_Z(l), b.get_Z(l)), (k, l)
        assert np.array_equal(a.get_U(), b.get_U())
        ta, tb = a.get_steps(), b.get_steps()
        assert all(np.array_equal(x, y) for x, y in zip(ta, tb))
    a.close()
    b.close()


def test_inference_matches_the_oracle_between_iterations():
    from paper_2112_09335_amd import binding
    w = synth.config(3, 0.01)
    solver = binding.Solver.from_workload(w, 0)
    orc = make_oracle(w)
    accs = []
    for k in range(0, 7):
        if k:
            solver.run(1)
            orc.iterate(1)
        pg, lg, ag = solver.predict()
        po, lo, ao = orc.predict()
        scale = np.abs(lo).max()
        assert np.abs(lg - lo).max() <= 1e-4 * scale
        top2 = np.sort(lo, axis=1)[:, -2:]
        clear = (top2[:, 1] - top2[:, 0]) > 1e-3 * scale          # rows whose class is not a near tie
        assert clear.mean() > 0.9
        assert np.array_equal(pg[clear], po[clear])
        assert abs(ag - ao) <= (~clear).mean() + 1e-12
        accs.append(ag)
        # predict leaves the iterate alone
        assert abs(solver.eval()["objective"] - orc.stats()["objective"]) <= 1e-4 * orc.stats()["objective"]
    say("accuracy per iteration", accs)
    solver.close()


def test_dual_ascent_on_new_iterates_variant():
    w = synth.config(1, 0.5)
    w.hyper["dual_form"] = 1
    run_case(w, 6, "dual-form-1")
    w = synth.config(3, 0.005)
    w.hyper["dual_form"] = 1
    run_case(w, 5, "dual-form-1/3-layer")


def test_low_rank_gradient_path_and_its_stored_twin():
    """Narrow next layers (multiples of four up to 16 units) keep the Z gradient in low-rank form; both that
    path and the stored-gradient path must match the oracle, three layers so that both hidden layers use it."""
    from paper_2112_09335_amd import binding
    w = synth.make_workload("lowrank", 21, 1500, 6, [36, 48, 12, 4], 4, 6, graph="sbm", features="gaussian",
                            avg_degree=9, frac_intra=0.8)
    run_case(w, 6, "low-rank")
    a = binding.Solver.from_workload(w, 0)
    b = binding.Solver.from_workload(w, 0)
    b.tune("use_lowrank", 0)
    a.run(5)
    b.run(5)
    for l in range(1, w.L + 1):
        za, zb = a.get_Z(l), b.get_Z(l)
        assert np.abs(za - zb).max() <= 1e-5 * np.abs(zb).max()
    ta, tb = a.get_steps(), b.get_steps()
    assert np.array_equal(ta[0], tb[0]) and np.array_equal(ta[1], tb[1]) and np.array_equal(ta[2], tb[2])
    a.close()
    b.close()


def test_layer_by_layer_schedule_matches_the_oracle():
    """Serial baseline of Section 4.1 (schedule 1): W_l then Z_l, layer after layer, newest values everywhere."""
    w = synth.config(1, 0.5)
    w.hyper["schedule"] = 1
    run_case(w, 8, "layer-by-layer/config1")
    w = synth.config(3, 0.01)                       # three layers: both kinds of hidden Z update
    w.hyper["schedule"] = 1
    run_case(w, 6, "layer-by-layer/config3")
    w = synth.config(4, 0.002)                      # narrow-side association, low-rank gradient, hub rows
    w.hyper["schedule"] = 1
    w.hyper["dual_form"] = 1
    run_case(w, 6, "layer-by-layer/config4/dual-form-1")
    w = synth.make_workload("serial", 14, 900, 1, [24, 40, 12, 5], 5, 5, graph="sbm", features="gaussian",
                            avg_degree=8, frac_intra=1.0)
    w.hyper["schedule"] = 1                         # the paper's serial run: one community
    run_case(w, 6, "layer-by-layer/one-community")


def test_step_parameters_that_may_shrink_again():
    """step_policy 1: every search starts one notch below the value accepted last time."""
    w = synth.config(1, 0.5)
    w.hyper["step_policy"] = 1
    run_case(w, 8, "step-policy-1/config1")
    w = synth.config(3, 0.01)
    w.hyper["step_policy"] = 1
    run_case(w, 6, "step-policy-1/config3")
    w = synth.config(4, 0.002)
    w.hyper["step_policy"] = 1
    w.hyper["schedule"] = 1
    run_case(w, 6, "step-policy-1/config4/layer-by-layer")


def test_fp32_matrix_core_path_matches_the_oracle_too():
    """The sweep with the wide products on the fp32 MFMA kernels (gemm_split = 0) instead of the bf16-split ones."""
    from paper_2112_09335_amd import binding
    w = synth.config(3, 0.01)
    probe = binding.Solver(device=-1)
    try:
        probe.tune("gemm_split", 0)              # process-wide switch
        run_case(w, 5, "fp32-mfma/config3")
    finally:
        probe.tune("gemm_split", 1)
        probe.close()


def test_hub_rows_and_hub_segments_are_split_inside_the_sweep():
    """Rows and (row, community) segments above the aggregation's split threshold (384 entries), as the power-law graph
    has them at full size, inside whole iterations: the aggregation that carries the penalty term nu (Z_l - relu(T_l))
    of the Z gradient (Appendix A, Eqs. 3, 4) on split rows and its combine kernel, the low-rank form of the gradient,
    the segment products of the theta search and the carried pre-activations."""
    base = synth.make_workload("hub", 31, 2400, 5, [24, 32, 32, 8], 8, 6, graph="sbm", features="gaussian",
                               avg_degree=8, frac_intra=0.8)
    w = synth.add_hubs(base, 32, 3, 700, 0.65)
    deg = np.bincount(w.src, minlength=w.N) + np.bincount(w.dst, minlength=w.N)
    assert np.sort(deg)[-3] > 500
    # layer 1: C_2 >= C_1, so G_2 W_2^T is aggregated at width 32 with the penalty epilogue; layer 2: low-rank form
    run_case(w, 6, "hubs/epilogue-aggregation+low-rank")
    # widths that are no multiple of four (one column per lane) through the same path
    base = synth.make_workload("hub", 33, 2000, 4, [20, 30, 30, 5], 5, 6, graph="sbm", features="gaussian",
                               avg_degree=8, frac_intra=0.8)
    run_case(synth.add_hubs(base, 34, 2, 600, 0.7), 5, "hubs/odd-widths")
    # two layers, narrow last layer: low-rank gradient and narrow-side association of layer 2 on hub rows
    base = synth.make_workload("hub", 35, 2400, 6, [24, 40, 8], 8, 6, graph="dcsbm", features="gaussian",
                               avg_degree=10, frac_intra=0.8, exponent=2.5)
    w = synth.add_hubs(base, 36, 3, 650, 0.7)
    run_case(w, 6, "hubs/low-rank-two-layers")
    run_case(w, 5, "hubs/stored-gradient-two-layers", tune=dict(use_lowrank=0))


def test_carried_pre_activations_across_their_refresh():
    """T_l = A~ Z_{l-1} W_l is carried from one iteration to the next by update formulas and formed anew every
    t1_refresh iterations: compare with the oracle at every age, across several refreshes, and over more than one
    full period of the default."""
    w = synth.config(1, 0.5)
    run_case(w, 11, "carry/config1/refresh4", tune=dict(t1_refresh=4))
    w = synth.config(3, 0.005)                       # three layers: T_2, T_3 carried through the Z steps
    run_case(w, 10, "carry/config3/refresh3", tune=dict(t1_refresh=3))
    w = synth.config(4, 0.002)                       # narrow-side association: the carried T_2 skips an aggregation
    run_case(w, 10, "carry/config4/refresh4", tune=dict(t1_refresh=4))
    w = synth.config(1)                              # default period of 16: ages 1..16, the refresh, and beyond
    run_case(w, 19, "carry/config1/default-period")
    w = synth.config(3, 0.005)
    run_case(w, 18, "carry/config3/default-period")


def test_last_layer_by_fista_with_backtracking():
    """fista_mode 1: Z_{L,m} by FISTA with backtracking on the block (one L per community and step, found on the device);
    iterates, the L every solve ends with and the number of candidates it tested must match the oracle."""
    w = synth.config(1, 0.5)
    w.hyper["fista_mode"] = 1
    run_case(w, 8, "fista-backtracking/config1")
    w = synth.config(3, 0.005)                       # three layers, ten classes
    w.hyper["fista_mode"] = 1
    run_case(w, 6, "fista-backtracking/config3")
    w = synth.make_workload("ragged", 11, 1237, 5, [37, 50, 9, 6], 6, 6, graph="sbm", features="gaussian",
                            avg_degree=6, frac_intra=0.7, labelled_fraction=0.4)
    w.comm = np.where(w.comm == 3, 4, w.comm).astype(np.int32)      # community 3 is empty; most rows have no label
    w.hyper["fista_mode"] = 1
    run_case(w, 5, "fista-backtracking/ragged-ce")
    w2 = copy.deepcopy(w)
    w2.hyper["risk"] = 1
    w2.hyper["dual_form"] = 1
    run_case(w2, 4, "fista-backtracking/ragged-lsq/dual-form-1")
    w = synth.config(4, 0.002)                       # 16 classes, 64 communities
    w.hyper["fista_mode"] = 1
    run_case(w, 4, "fista-backtracking/config4")
    # a cap on the multiplications that binds: L cannot reach the curvature, both sides must raise the status bit (the
    # solve then overshoots and the iteration amplifies rounding within a few iterations, so only two are compared)
    w.hyper["max_backtrack"] = 6
    run_case(w, 2, "fista-backtracking/config4/cap")
    w = synth.make_workload("wide-last", 41, 900, 3, [20, 24, 40], 40, 4, graph="sbm", features="gaussian",
                            avg_degree=8, frac_intra=0.8)   # 40 classes: sixteen lanes per row
    w.hyper["fista_mode"] = 1
    w.hyper["schedule"] = 1
    run_case(w, 4, "fista-backtracking/40-classes/layer-by-layer")


def test_more_communities_than_a_workgroup_keeps_step_parameters_for():
    """The Z-step and carry kernels keep 1/theta of up to 1024 communities in LDS and look the parameters up in memory
    beyond that: 1100 communities of a few nodes each, on the low-rank path (two layers) and on the stored-gradient
    path (three layers)."""
    run_case(synth.config(4, 0.002, M=1100), 3, "many-communities/config4")       # N = 4000
    run_case(synth.config(3, 0.008, M=1100), 3, "many-communities/config3")       # N = 1600, three layers


def test_communities_from_the_library_partitioner_feed_the_sweep():
    """A graph that comes without communities: cadmm_partition (bit-exact against its CPU twin) supplies them, the graph
    built from them is bit-exact against the oracle's, and the sweep on them matches the oracle iteration by iteration."""
    from oracle.graph import OracleGraph
    from oracle.partition import partition as twin_partition
    from paper_2112_09335_amd import binding
    w = synth.config(2, 0.1)                          # N = 2000, planted blocks thrown away
    host = binding.Solver(device=-1)
    comm = host.partition(w.N, w.src, w.dst, w.M)
    host.close()
    assert np.array_equal(comm, np.asarray(twin_partition(w.N, w.src, w.dst, w.M), dtype=np.int32))
    assert comm.min() >= 0 and comm.max() < w.M and not np.array_equal(comm, w.comm)
    w.comm = comm
    s = binding.Solver.from_workload(w, 0)
    g = s.get_graph()
    og = OracleGraph(w.N, w.src, w.dst, w.M, w.comm)
    assert np.array_equal(g["perm"], og.perm) and np.array_equal(g["row_ptr"], og.row_ptr)
    assert np.array_equal(g["col"], og.col) and np.array_equal(g["val"], og.val.astype(np.float32))
    assert np.array_equal(g["seg_ptr"], og.seg_ptr) and np.array_equal(g["seg_comm"], og.seg_comm)
    assert np.array_equal(g["neighbour"], og.neighbour)
    s.close()
    run_case(w, 6, "library-partitioner/config2")
