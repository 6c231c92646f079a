"""Helpers shared by the GPU parity tests: tolerances and the oracle <-> library comparison."""
import json
import os
import sys
import time

import numpy as np

REL = 1e-4      # tolerance stated for W, Z, U and the objective (fp32 state vs the fp64 oracle)

# One record per parity case (ties used, worst error): kept for the summary that conftest.py prints at the end of a
# run (also under -q) and appended to a JSON-lines file that survives the run.
CASE_RECORDS = []
CASE_LOG = os.environ.get("CADMM_PARITY_LOG", os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))),
                                                           "gpurun_out", "parity_cases.jsonl"))


def record_case(**rec):
    rec["time"] = time.strftime("%Y-%m-%dT%H:%M:%S")
    CASE_RECORDS.append(rec)
    try:
        os.makedirs(os.path.dirname(CASE_LOG), exist_ok=True)
        with open(CASE_LOG, "a") as f:
            f.write(json.dumps(rec) + "\n")
    except OSError:
        pass                    # a read-only tree loses the file, not the summary


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def close(name, got, ref, floor=0.0):
    """Relative Frobenius error and max-abs error, both against REL (plus an absolute floor for
    quantities that are differences of much larger ones)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (name, got.shape, ref.shape)
    assert np.all(np.isfinite(got)), name
    err = np.abs(got - ref)
    fro = np.linalg.norm(got - ref)
    assert fro <= REL * np.linalg.norm(ref) + floor * np.sqrt(ref.size), \
        f"{name}: rel Frobenius error {fro / max(np.linalg.norm(ref), 1e-300):.3e}"
    assert err.max(initial=0.0) <= REL * np.abs(ref).max(initial=0.0) + floor, \
        f"{name}: max abs error {err.max():.3e} vs max |ref| {np.abs(ref).max():.3e}"
    return fro / max(np.linalg.norm(ref), 1e-300)


# A pre-activation counts as tied if its fp64 value is within this many units of the rms of its layer block:
# 16 fp32 roundings (16 * 2^-24), which covers the rounding of a contraction over a few hundred terms in fp32 and
# the drift of pre-activations that are carried by update formulas for up to 16 iterations.  The largest |T| / rms
# of a tie seen over all parity cases is 3.7e-7.
TIE_BAND = 1e-6
# Entries of a hidden pre-activation that an fp32 implementation may put on the other side of zero, per entry and
# evaluation: those within its rounding error delta of zero, about 0.8 * delta / rms for a bell-shaped distribution
# (density 0.4 / rms at zero, both sides), with delta = 3e-7 rms as measured.
TIE_RATE = 0.8 * 3e-7


def expected_ties(N, dims, iters):
    """Expected number of tied entries in `iters` iterations: an iteration looks at ReLU'(T_l) for l = 1..L-1 in
    the W step and again, after the W step, for l = 2..L-1 in the Z step of layer l-1."""
    L = len(dims) - 1
    entries = sum(N * dims[l] for l in range(1, L)) + sum(N * dims[l] for l in range(2, L))
    return TIE_RATE * entries * iters
MAX_TIE_CANDIDATES = 8      # entries inside the band in one iteration; more would make the band unselective
MAX_TIE_FLIPS = 2           # entries of one iteration allowed to fall on the other side


def step_with_relu_ties(solver, orc, tag):
    """One more iteration on both sides, then compare.  If they disagree, ask whether a ReLU tie explains it: the
    gradient of the penalty nu/2 ||Z - relu(T)||^2 jumps where a pre-activation T crosses 0, so an entry that is
    zero up to fp32 rounding may fall on either side, and both outcomes are valid iterates.  The oracle's iteration
    is repeated from the same state while it records the entries of its fp64 pre-activations with
    |T| <= TIE_BAND * rms(T); then it is repeated with the derivative of at most MAX_TIE_FLIPS of exactly those
    entries taken on the other side (every other entry keeps ReLU'(T) = 1[T > 0]); the GPU result must match one of
    these outcomes to the same tolerance.  Returns (worst relative error, list of flipped entries)."""
    import oracle.admm as oa
    hook = oa.RELU_TIES
    snap = orc.snapshot()
    solver.run(1)
    orc.iterate(1)
    try:
        return compare_iterate(solver, orc, tag), []
    except AssertionError as first:
        try:
            orc.restore(snap)
            hook.reset()
            hook.band = TIE_BAND
            orc.iterate(1)
            cands = sorted(hook.found.items(), key=lambda kv: kv[1][0])
            say(f"{tag}: mismatch ({str(first).splitlines()[0][:140]}); pre-activations within {TIE_BAND:g} rms of "
                f"zero: {[(k, f'{v[0]:.1e}') for k, v in cands]}")
            assert len(cands) <= MAX_TIE_CANDIDATES, f"{tag}: {len(cands)} entries inside the tie band"
            keys = [k for k, _ in cands]
            subsets = [(k,) for k in keys]
            if MAX_TIE_FLIPS >= 2:
                subsets += [(a, b) for i, a in enumerate(keys) for b in keys[i + 1:]]
            for sub in subsets:
                orc.restore(snap)
                hook.reset()
                hook.band = TIE_BAND
                hook.flips = set(sub)
                orc.iterate(1)
                if set(hook.flipped) != set(sub):
                    continue            # the flipped W step moved an entry of the Z step out of the band
                try:
                    worst = compare_iterate(solver, orc, tag + f" [relu tie {sub}]")
                except AssertionError:
                    continue
                used = [dict(step=k[0], layer=k[1], row=k[2], col=k[3], abs_over_rms=hook.flipped[k]) for k in sub]
                say(f"{tag}: ReLU tie, matches the oracle with the derivative flipped at {used}")
                return worst, used
            raise first
        finally:
            hook.reset()


def compare_iterate(solver, orc, tag):
    """W, Z, U, objective, residuals and the step-size trajectory after one more iteration."""
    L = orc.L
    zl_scale = float(np.abs(orc.Z[L]).max())
    worst = 0.0
    for l in range(1, L + 1):
        worst = max(worst, close(f"{tag} W{l}", solver.get_W(l), orc.get_W(l)))
        worst = max(worst, close(f"{tag} Z{l}", solver.get_Z(l), orc.get_Z(l)))
    close(f"{tag} U", solver.get_U(), orc.get_U(), floor=1e-9 * zl_scale)
    sg, so = solver.eval(), orc.stats()
    for key in ("objective", "lagrangian", "risk", "primal_res"):
        assert abs(sg[key] - so[key]) <= REL * abs(so[key]) + 1e-9 * zl_scale, (tag, key, sg[key], so[key])
    assert abs(sg["dual_res"] - so["dual_res"]) <= REL * abs(so["dual_res"]) + 1e-7 * zl_scale * orc.rho, \
        (tag, "dual_res", sg["dual_res"], so["dual_res"])
    for a, b in zip(sg["layer_penalty"], so["layer_penalty"]):
        assert abs(a - b) <= REL * abs(b) + 1e-12 * max(so["objective"], 1.0), (tag, "penalty", a, b)
    assert sg["iter"] == so["iter"]
    assert sg["status"] == so["status"], (tag, "status", sg["status"], so["status"])
    # step-size trajectory: identical values, except where the decision was taken on a gradient that is
    # zero up to rounding on both sides (then the block does not move and the value is immaterial)
    tau_g, theta_g, tr_g, g_g = solver.get_steps()
    tau_o, theta_o, tr_o = orc.get_steps()
    step_g = np.concatenate([tau_g, theta_g])
    step_o = np.concatenate([tau_o, theta_o])
    differ = (step_g != step_o) | (tr_g != tr_o)
    assert not np.any(differ & (g_g > 1e-20)), (tag, "steps", step_g[differ], step_o[differ], tr_g[differ], tr_o[differ])
    if getattr(orc, "fista_mode", 0) == 1 and orc.k > 0:
        # last layer with backtracking: the constant every community's solve ended with and the candidates it tested
        L_g, tr_g = solver.get_fista()
        assert np.array_equal(L_g, np.array(orc.fista_L)), (tag, "fista L", L_g, orc.fista_L)
        assert np.array_equal(tr_g, np.array(orc.fista_trials, dtype=np.int32)), (tag, "fista trials", tr_g, orc.fista_trials)
    return worst
