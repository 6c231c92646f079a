"""Helpers shared by the GPU parity tests: tolerances and the oracle <-> library comparison."""
import sys

import numpy as np

REL = 1e-4      # tolerance stated for W, Z, U and the objective (fp32 state vs the fp64 oracle)


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


def step_with_relu_ties(solver, orc, tag):
    """One more iteration on both sides, then compare.  If they disagree, ask whether a ReLU tie explains
    it: the gradient of the penalty nu/2 ||Z - relu(T)||^2 jumps where a pre-activation T crosses 0, so
    an entry that is zero up to fp32 rounding may fall on either side.  The oracle's iteration is
    repeated from the same state with the threshold of ReLU' moved by +-delta (a few fp32 roundings of
    the pre-activation scale), separately for the W step and the Z step, which look at different
    pre-activations; the GPU result must then match one of these equally valid outcomes to the same
    tolerance.  Returns (worst relative error, tie used?)."""
    import oracle.admm as oa
    snap = orc.snapshot()
    solver.run(1)
    orc.iterate(1)
    try:
        return compare_iterate(solver, orc, tag), False
    except AssertionError as first:
        # fp32 rounding of a pre-activation of size ~scale is a few 1e-7 * scale; a finer-to-coarser ladder
        # so that only the entry nearest to zero changes side first
        scale = max(1.0, max(float(np.sqrt(np.mean(z * z))) for z in snap["Z"][1:]))
        rungs = [0.0] + [sgn * m * 1e-7 * scale for m in (0.1, 0.3, 1, 2, 4, 8, 16, 32) for sgn in (+1, -1)]
        pairs = sorted(((a, b) for a in rungs for b in rungs if (a, b) != (0.0, 0.0)),
                       key=lambda p: ((p[0] != 0.0) + (p[1] != 0.0), abs(p[0]) + abs(p[1])))
        for shift_w, shift_z in pairs:
            orc.restore(snap)
            oa.RELU_TIE_SHIFT["W"], oa.RELU_TIE_SHIFT["Z"] = shift_w, shift_z
            try:
                orc.iterate(1)
            finally:
                oa.RELU_TIE_SHIFT["W"], oa.RELU_TIE_SHIFT["Z"] = 0.0, 0.0
            try:
                worst = compare_iterate(solver, orc, tag + f" [relu tie shifts {shift_w:+.1e} {shift_z:+.1e}]")
                say(f"{tag}: ReLU tie, matches the oracle with thresholds W {shift_w:+.2e}, Z {shift_z:+.2e}; "
                    f"first mismatch was: {str(first).splitlines()[0][:160]}")
                return worst, True
            except AssertionError:
                continue
        raise first


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
    return worst
