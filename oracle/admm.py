"""CPU oracle, part 2: the community-based ADMM sweep.  TEST INFRASTRUCTURE ONLY.

Plain numpy in fp64, written step by step from the paper (Section 3 and Appendix A)
in its notation: first-order messages p, second-order messages s, the subproblem
objectives phi (W) and psi (Z), their quadratic models P and Q with backtracking on
tau_l and theta_{l,m}, FISTA for the last layer, the dual step.  It shares no code
with the HIP library and must never be imported by the product path.

Everything is held in the community-contiguous node order of ``OracleGraph``; a
"block" Z_{l,m} is the row range ``graph.rows(m)``.

Readings taken where the paper is silent (all are definitions of this build, so the
constants eta, tau0, theta0, J and the FISTA step are "parity unpinned" by the paper;
only oracle <-> GPU agreement and the invariants in the tests hold them):
  * initial point: W given, Z_l = forward pass, U = 0;
  * backtracking: start from the last accepted value (tau0 / theta0 at k = 0), multiply
    by eta until  model >= objective  holds (equality accepts), at most max_backtrack
    multiplications (then the step is taken anyway and a status bit is raised);
  * step_policy 1 lets the parameters shrink again: a search then starts from (last accepted value) / eta
    instead of the last accepted value itself (policy 0, the monotone choice above);
  * a step below resolution is not taken: if the first candidate would move the block by
    less than 1e-12 of its own norm, i.e. ||grad||^2 <= (1e-12 * tau)^2 * ||block||^2, the
    block keeps its value and its step parameter and no trial is counted (at the
    forward-pass initial point every hidden-layer gradient is zero up to rounding, and a
    search decided by rounding noise would inflate tau / theta arbitrarily);
  * ReLU'(0) = 0;
  * R = softmax cross-entropy summed over labelled rows (risk 0) or
    1/2 ||Z_L - Y||^2 over labelled rows (risk 1); unlabelled rows contribute nothing;
  * last layer: J FISTA steps of size 1/(rho + c_R) from the current Z_L
    (c_R = 1/2 for cross-entropy, 1 for least squares bounds the Hessian of R);
    a row without label has the exact minimiser  b = c - U/rho  of its quadratic;
  * fista_mode 1 is FISTA with backtracking (the second form Beck and Teboulle give) on the block subproblem of
    Z_{L,m} (Eq. 5): one constant L per community and step, started at L = rho in every ADMM iteration (the curvature
    of the quadratic part, a lower bound of every curvature of the objective), multiplied by eta until
    F(y - grad/L) <= F(y) - ||grad||^2 / (2L)  (the condition F(p_L(y)) <= Q_L(p_L(y), y) without a non-smooth term;
    equality up to 1e-12 |F(y)| accepts, so that the rounding of F does not decide a search near the solution),
    at most max_backtrack multiplications per step, and kept for the later steps of the same solve; a step below
    resolution (||grad||^2 <= (1e-12 L)^2 ||y||^2) is not taken, as for W and Z; rows without label are outside
    the sums and take their exact minimiser as in mode 0;
  * dual step with the superscripts as printed (Eq. 2): Z_L^k and p^k (p uses W^{k+1}); dual_form = 1
    selects the usual ADMM dual ascent on the new iterates (Z_L^{k+1}, Z_{L-1}^{k+1}, W_L^{k+1}) instead;
  * updates are Jacobi: W^{k+1} from (W^k, Z^k, U^k); every Z^{k+1}_{l,m} from
    (W^{k+1}, Z^k, U^k)  (schedule 0, Algorithm 1 as printed);
  * schedule 1 is the serial baseline of Section 4.1 ("layers trained sequentially"), read as a
    Gauss-Seidel pass over the layers: for l = 1..L first W_l, then Z_l (all communities of the layer
    together), each from the newest values of everything else, i.e. W_l from (Z_{l-1}^{k+1}, Z_l^k),
    Z_l from (W_l^{k+1}, Z_{l-1}^{k+1}, W_{l+1}^k, Z_{l+1}^k); the dual step closes the pass and
    follows dual_form, where "Z_{L-1}^k" of form 0 is the Z_{L-1} the last-layer update saw.
"""
from __future__ import annotations

import numpy as np

from .graph import OracleGraph


def relu(x):
    return np.maximum(x, 0.0)


# ReLU'(x) = 1[x > 0] (the reading ReLU'(0) = 0).  The derivative of the penalty nu/2 ||Z - relu(T)||^2 jumps where a
# pre-activation T crosses 0, so an entry whose fp64 value is zero up to the fp32 rounding of the contraction that
# forms it may fall on either side in an fp32 implementation, and both outcomes are valid iterates.  The tests use
# this hook to make such a tie checkable entry by entry: with ``band`` > 0 every evaluation of ReLU' records the
# entries with |T| <= band * rms(T of that block), keyed by (step, layer of T, row, column); ``flips`` names entries
# whose derivative is to be taken on the other side, and only entries inside the band may be named.  The W step
# and the Z step of one iteration look at different pre-activations (before and after the W step), hence the step
# in the key.  With band = 0 and no flips (the default) this is the plain definition.
class ReluTieHook:
    def __init__(self):
        self.reset()

    def reset(self):
        self.band = 0.0
        self.found = {}       # key -> (|T| / rms, T): the candidates seen with band > 0
        self.flips = set()    # keys whose derivative is flipped
        self.flipped = {}     # key -> |T| / rms of the flips that were applied


RELU_TIES = ReluTieHook()


def relu_grad(x, step="W", layer=0, rows=None):
    mask = (x > 0.0).astype(np.float64)
    hook = RELU_TIES
    if hook.band <= 0.0 or x.size == 0:
        return mask
    scale = float(np.sqrt(np.mean(x * x)))
    r0 = 0 if rows is None else rows.start
    near = np.argwhere(np.abs(x) <= hook.band * scale)
    for i, j in near:
        key = (step, int(layer), int(r0 + i), int(j))
        rel = abs(float(x[i, j])) / scale if scale > 0 else 0.0
        hook.found[key] = (rel, float(x[i, j]))
        if key in hook.flips:
            mask[i, j] = 1.0 - mask[i, j]
            hook.flipped[key] = rel
    return mask


def inner(a, b):
    return float(np.sum(a * b))


def sqnorm(a):
    return float(np.sum(a * a))


def fista_rows(z0, c, u, y, lab, rho, J, risk):
    """J FISTA steps per row on  R(z, y) + <u, z - c> + rho/2 ||z - c||^2  from z0 (Appendix A, Eq. 5).
    The smooth part is the whole objective, so x_j = y_j - grad(y_j)/Lip with the usual momentum; rows
    without label take the exact minimiser c - u/rho of their quadratic."""
    Lip = rho + (0.5 if risk == 0 else 1.0)

    def grad(z):
        g = u + rho * (z - c)
        zl = z[lab]
        if risk == 0:
            e = np.exp(zl - zl.max(axis=1, keepdims=True))
            g[lab] += e / e.sum(axis=1, keepdims=True) - y[lab]
        else:
            g[lab] += zl - y[lab]
        return g

    x_prev = z0.copy()
    yk = x_prev.copy()
    t = 1.0
    x = x_prev
    for _ in range(J):
        x = yk - grad(yk) / Lip
        t_next = 0.5 * (1.0 + np.sqrt(1.0 + 4.0 * t * t))
        yk = x + ((t - 1.0) / t_next) * (x - x_prev)
        x_prev, t = x, t_next
    x = x.copy()
    x[~lab] = (c - u / rho)[~lab]
    return x


class AdmmOracle:
    STATUS_BACKTRACK_CAP = 1
    STATUS_NONFINITE = 2
    STEP_FLOOR = 1e-12
    FISTA_SLACK = 1e-12       # the backtracking test of fista_mode 1 accepts up to this relative rounding of F

    def __init__(self, graph: OracleGraph, dims, *, nu, rho, tau0, theta0, eta, max_backtrack,
                 fista_iters, risk=0, dual_form=0, schedule=0, step_policy=0, fista_mode=0):
        self.g = graph
        self.M = graph.M
        self.N = graph.N
        self.dims = [int(c) for c in dims]
        self.L = len(self.dims) - 1
        if self.L < 2:
            raise ValueError("need at least two layers")
        # hyper-parameters travel as fp32 at the library boundary; take exactly those values
        f32 = lambda v: float(np.float32(v))
        self.nu, self.rho, self.eta = f32(nu), f32(rho), f32(eta)
        self.tau = [None] + [f32(tau0)] * self.L                          # tau[l], l = 1..L
        self.theta = [None] + [[f32(theta0)] * self.M for _ in range(self.L - 1)]   # theta[l][m], l = 1..L-1
        self.max_backtrack = int(max_backtrack)
        self.J = int(fista_iters)
        self.risk = int(risk)
        self.dual_form = int(dual_form)
        if self.dual_form not in (0, 1):
            raise ValueError("dual_form must be 0 (Eq. 2 as printed) or 1 (new iterates)")
        self.step_policy = int(step_policy)
        if self.step_policy not in (0, 1):
            raise ValueError("step_policy must be 0 (start from the last accepted value) or 1 (from that / eta)")
        self.fista_mode = int(fista_mode)
        if self.fista_mode not in (0, 1):
            raise ValueError("fista_mode must be 0 (constant step) or 1 (backtracking)")
        self.fista_L = [0.0] * self.M          # L of the last FISTA step per community (mode 1)
        self.fista_trials = [0] * self.M       # candidates tested in the last solve per community (mode 1)
        self.schedule = int(schedule)
        if self.schedule not in (0, 1):
            raise ValueError("schedule must be 0 (Algorithm 1) or 1 (layer by layer)")
        self.block_trace = None       # a list here receives (name, l, L_rho) after every primal block update of schedule 1
        self.k = 0
        self.status = 0
        self.trials_W = [0] * (self.L + 1)
        self.trials_Z = [None] + [[0] * self.M for _ in range(self.L - 1)]
        self.TL_prev = None

    # ------------------------------------------------------------------ data / init
    def set_data(self, X_old, labels_old):
        self.Z = [None] * (self.L + 1)
        self._AZ0 = None
        self.Z[0] = self.g.to_new(np.asarray(X_old, dtype=np.float64))
        self.labels = self.g.to_new(np.asarray(labels_old, dtype=np.int64))
        CL = self.dims[-1]
        if self.labels.max(initial=-1) >= CL:
            raise ValueError("label out of range")
        self.Y = np.zeros((self.N, CL))
        lab = self.labels >= 0
        self.Y[np.flatnonzero(lab), self.labels[lab]] = 1.0
        self.labelled = lab

    def init(self, W0):
        """W given; Z_l = f_l(A~ Z_{l-1} W_l), Z_L = A~ Z_{L-1} W_L (constraints of Problem 1); U = 0."""
        self.W = [None] + [np.asarray(w, dtype=np.float64).copy() for w in W0]
        for l in range(1, self.L + 1):
            assert self.W[l].shape == (self.dims[l - 1], self.dims[l])
            T = np.vstack([self.g.aggregate_block(m, self.Z[l - 1]) @ self.W[l] for m in range(self.M)])
            self.Z[l] = relu(T) if l < self.L else T
        self.U = np.zeros((self.N, self.dims[-1]))
        self.k = 0
        self.TL_prev = None

    def blk(self, X, m):
        return X[self.g.rows(m)]

    # ------------------------------------------------------------------ risk R(Z_L, Y)
    def risk_value(self, ZL_rows, Y_rows, lab_rows):
        """R restricted to some rows (it is a sum over labelled rows)."""
        z = ZL_rows[lab_rows]
        y = Y_rows[lab_rows]
        if z.shape[0] == 0:
            return 0.0
        if self.risk == 0:
            zmax = z.max(axis=1, keepdims=True)
            lse = zmax[:, 0] + np.log(np.sum(np.exp(z - zmax), axis=1))
            return float(np.sum(lse - np.sum(y * z, axis=1)))
        return 0.5 * sqnorm(z - y)

    def risk_grad(self, z, y):
        """dR/dz for labelled rows."""
        if self.risk == 0:
            e = np.exp(z - z.max(axis=1, keepdims=True))
            return e / e.sum(axis=1, keepdims=True) - y
        return z - y

    # ------------------------------------------------------------------ phi  (Section 3, definitions of phi)
    def phi(self, l, Wl, Zprev, Zl, U=None):
        """phi(W_l, Z_{l-1}, Z_l) for l < L, phi(W_L, Z_{L-1}, Z_L, U) for l = L, in the blocked form."""
        tot = 0.0
        for m in range(self.M):
            T = self.g.aggregate_block(m, Zprev) @ Wl
            if l < self.L:
                tot += 0.5 * self.nu * sqnorm(self.blk(Zl, m) - relu(T))
            else:
                r = self.blk(Zl, m) - T
                tot += inner(self.blk(U, m), r) + 0.5 * self.rho * sqnorm(r)
        return tot

    def grad_phi_W(self, l, Wl, Zprev, Zl, U=None):
        """Gradient of phi with respect to W_l."""
        g = np.zeros_like(Wl)
        for m in range(self.M):
            H = self.g.aggregate_block(m, Zprev)
            T = H @ Wl
            if l < self.L:
                G = self.nu * (relu(T) - self.blk(Zl, m)) * relu_grad(T, "W", l, self.g.rows(m))
            else:
                r = self.blk(Zl, m) - T
                G = -(self.blk(U, m) + self.rho * r)
            g += H.T @ G
        return g

    # ------------------------------------------------------------------ W-update (Section 3.1)
    def update_W(self, l, Wk, Zk, Uk):
        """W_l^{k+1} = argmin P_l(W; tau): a gradient step of length 1/tau, tau found by backtracking
        until  P_l(W^{k+1}; tau) >= phi(W^{k+1}, Z^k_{l-1}, Z^k_l (, U^k))."""
        W = Wk[l]
        phi0 = self.phi(l, W, Zk[l - 1], Zk[l], Uk)
        grad = self.grad_phi_W(l, W, Zk[l - 1], Zk[l], Uk)
        tau = self.tau[l] / self.eta if self.step_policy == 1 else self.tau[l]
        trials = 0
        if sqnorm(grad) <= (self.STEP_FLOOR * tau) ** 2 * sqnorm(W):
            self.trials_W[l] = 0
            return W.copy()
        while True:
            Wn = W - grad / tau
            model = phi0 + inner(grad, Wn - W) + 0.5 * tau * sqnorm(Wn - W)
            trials += 1
            if self.phi(l, Wn, Zk[l - 1], Zk[l], Uk) <= model:
                break
            if trials > self.max_backtrack:
                self.status |= self.STATUS_BACKTRACK_CAP
                break
            tau *= self.eta
        self.tau[l] = tau
        self.trials_W[l] = trials
        return Wn

    # ------------------------------------------------------------------ messages (Appendix A)
    def first_order(self, l, Zl, Wnext):
        """p_{l, r->m} = A~_{m,r} Z_{l,r} W_{l+1}  for every m and r in N_m or r = m.  Key (r, m)."""
        p = {}
        for r in range(self.M):
            ZW = self.blk(Zl, r) @ Wnext
            for m in self.g.nbr_and_self(r):          # r in N_m  <=>  m in N_r (undirected graph)
                p[(r, m)] = self.g.block[(m, r)] @ ZW
        return p

    def second_order(self, l, p_l, Znext, U):
        """s_{l, r->m} = [s1, s2] for r in N_m (Appendix A, second-order information).

        l <= L-2:  s1 = Z_{l+1,r},                                   s2 = sum_{r' in N_r u {r} minus {m}} p_{l,r'->r}
        l  = L-1:  s1 = Z_{L,r} - sum_{r' in N_r u {r} minus {m}} p_{L-1,r'->r},   s2 = U_r
        """
        s = {}
        for m in range(self.M):
            for r in self.g.nbrs(m):
                acc = np.zeros_like(p_l[(r, r)])
                for rp in self.g.nbr_and_self(r):
                    if rp != m:
                        acc = acc + p_l[(rp, r)]
                if l <= self.L - 2:
                    s[(r, m)] = (self.blk(Znext, r), acc)
                else:
                    s[(r, m)] = (self.blk(Znext, r) - acc, self.blk(U, r))
        return s

    # ------------------------------------------------------------------ psi  (Appendix A, Eqs. 3, 4)
    def psi(self, l, m, Zlm, Wnext, Znext, U, p_prev, p_cur, s_cur):
        """Objective of the Z_{l,m} subproblem, l = 1..L-1, in the message form."""
        g = self.g
        own_pre = sum(p_prev[(r, m)] for r in g.nbr_and_self(m))
        val = 0.5 * self.nu * sqnorm(Zlm - relu(own_pre))
        a = g.block[(m, m)] @ Zlm @ Wnext
        for r in g.nbrs(m):
            a = a + p_cur[(r, m)]
        if l <= self.L - 2:
            val += 0.5 * self.nu * sqnorm(self.blk(Znext, m) - relu(a))
            for r in g.nbrs(m):
                s1, s2 = s_cur[(r, m)]
                val += 0.5 * self.nu * sqnorm(s1 - relu(g.block[(r, m)] @ Zlm @ Wnext + s2))
        else:
            res = self.blk(Znext, m) - a
            val += inner(self.blk(U, m), res) + 0.5 * self.rho * sqnorm(res)
            for r in g.nbrs(m):
                s1, s2 = s_cur[(r, m)]
                d = s1 - g.block[(r, m)] @ Zlm @ Wnext
                val += inner(s2, d) + 0.5 * self.rho * sqnorm(d)
        return val

    def grad_psi(self, l, m, Zlm, Wnext, Znext, U, p_prev, p_cur, s_cur):
        """Gradient of psi with respect to Z_{l,m}."""
        g = self.g
        own_pre = sum(p_prev[(r, m)] for r in g.nbr_and_self(m))
        grad = self.nu * (Zlm - relu(own_pre))
        a = g.block[(m, m)] @ Zlm @ Wnext
        for r in g.nbrs(m):
            a = a + p_cur[(r, m)]
        if l <= self.L - 2:
            Gm = self.nu * (relu(a) - self.blk(Znext, m)) * relu_grad(a, "Z", l + 1, g.rows(m))
            grad = grad + g.block[(m, m)].T @ Gm @ Wnext.T
            for r in g.nbrs(m):
                s1, s2 = s_cur[(r, m)]
                b = g.block[(r, m)] @ Zlm @ Wnext + s2
                Gr = self.nu * (relu(b) - s1) * relu_grad(b, "Z", l + 1, g.rows(r))
                grad = grad + g.block[(r, m)].T @ Gr @ Wnext.T
        else:
            res = self.blk(Znext, m) - a
            Gm = -(self.blk(U, m) + self.rho * res)
            grad = grad + g.block[(m, m)].T @ Gm @ Wnext.T
            for r in g.nbrs(m):
                s1, s2 = s_cur[(r, m)]
                d = s1 - g.block[(r, m)] @ Zlm @ Wnext
                Gr = -(s2 + self.rho * d)
                grad = grad + g.block[(r, m)].T @ Gr @ Wnext.T
        return grad

    def update_Z_hidden(self, l, m, Zk, Wn, Uk, p_prev, p_cur, s_cur):
        """Z_{l,m}^{k+1} = argmin Q_{l,m}(Z; theta): a gradient step of length 1/theta with backtracking
        until  Q_{l,m}(Z^{k+1}; theta) >= psi(Z^{k+1}, ...)   (Appendix A, Eqs. 6-8)."""
        Z = self.blk(Zk[l], m)
        args = (Wn[l + 1], Zk[l + 1], Uk, p_prev, p_cur, s_cur)
        psi0 = self.psi(l, m, Z, *args)
        grad = self.grad_psi(l, m, Z, *args)
        theta = self.theta[l][m] / self.eta if self.step_policy == 1 else self.theta[l][m]
        trials = 0
        if sqnorm(grad) <= (self.STEP_FLOOR * theta) ** 2 * sqnorm(Z):
            self.trials_Z[l][m] = 0
            return Z.copy()
        while True:
            Zn = Z - grad / theta
            model = psi0 + inner(grad, Zn - Z) + 0.5 * theta * sqnorm(Zn - Z)
            trials += 1
            if self.psi(l, m, Zn, *args) <= model:
                break
            if trials > self.max_backtrack:
                self.status |= self.STATUS_BACKTRACK_CAP
                break
            theta *= self.eta
        self.theta[l][m] = theta
        self.trials_Z[l][m] = trials
        return Zn

    # ------------------------------------------------------------------ last layer (Appendix A, Eq. 5)
    def psi_last(self, m, ZLm, Uk, p_last):
        c = sum(p_last[(r, m)] for r in self.g.nbr_and_self(m))
        rows = self.g.rows(m)
        return (self.risk_value(ZLm, self.Y[rows], self.labelled[rows])
                + inner(self.blk(Uk, m), ZLm - c) + 0.5 * self.rho * sqnorm(ZLm - c))

    def update_Z_last(self, m, Zk, Uk, p_last, J=None):
        """Z_{L,m}^{k+1}: FISTA on Eq. 5, whose smooth part is the whole objective (no non-smooth term),
        so the proximal map is the identity: x_j = y_j - grad(y_j)/Lip, with the usual momentum."""
        J = self.J if J is None else J
        rows = self.g.rows(m)
        c = sum(p_last[(r, m)] for r in self.g.nbr_and_self(m))
        if self.fista_mode == 1:
            return self.fista_block_backtracking(m, self.blk(Zk[self.L], m), c, self.blk(Uk, m), J)
        return fista_rows(self.blk(Zk[self.L], m), c, self.blk(Uk, m), self.Y[rows], self.labelled[rows],
                          self.rho, J, self.risk)

    def fista_block_backtracking(self, m, z0, c, u, J):
        """FISTA with backtracking on  F(Z) = R(Z, Y_m) + <U_m, Z - c> + rho/2 ||Z - c||^2  over the labelled rows of
        community m (Appendix A, Eq. 5; F is smooth, so the proximal map is the identity and a step is
        x = y - grad F(y) / L).  L starts at rho, grows by eta until F(x) <= F(y) - ||grad||^2 / (2L) (up to the
        rounding slack), and is kept for the later steps.  Rows without label take the exact minimiser c - u/rho of their quadratic."""
        rows = self.g.rows(m)
        lab = self.labelled[rows]
        Y = self.Y[rows][lab]
        cl, ul = c[lab], u[lab]

        def F(z):
            return (self.risk_value(z, Y, np.ones(z.shape[0], dtype=bool)) + inner(ul, z - cl)
                    + 0.5 * self.rho * sqnorm(z - cl))

        def grad(z):
            return ul + self.rho * (z - cl) + (self.risk_grad(z, Y) if z.shape[0] else 0.0)

        L = self.rho
        x_prev = z0[lab].copy()
        yk = x_prev.copy()
        x = x_prev
        t = 1.0
        total = 0
        for _ in range(J):
            if yk.shape[0] == 0:
                break
            Fy, g = F(yk), grad(yk)
            gg = sqnorm(g)
            trials = 0
            if gg <= (self.STEP_FLOOR * L) ** 2 * sqnorm(yk):     # a step below resolution is not taken
                x = yk
                t_next = 0.5 * (1.0 + np.sqrt(1.0 + 4.0 * t * t))
                yk = x + ((t - 1.0) / t_next) * (x - x_prev)
                x_prev, t = x, t_next
                continue
            while True:
                x = yk - g / L
                trials += 1
                if F(x) <= Fy - gg / (2.0 * L) + self.FISTA_SLACK * abs(Fy):
                    break
                if trials > self.max_backtrack:
                    self.status |= self.STATUS_BACKTRACK_CAP
                    break
                L *= self.eta
            total += trials
            t_next = 0.5 * (1.0 + np.sqrt(1.0 + 4.0 * t * t))
            yk = x + ((t - 1.0) / t_next) * (x - x_prev)
            x_prev, t = x, t_next
        self.fista_L[m] = L
        self.fista_trials[m] = total
        out = (c - u / self.rho).copy()
        out[lab] = x
        return out

    # ------------------------------------------------------------------ one iteration of Algorithm 1
    def iterate(self, k=1):
        for _ in range(k):
            if self.schedule == 0:
                self._sweep()
            else:
                self._sweep_layer_by_layer()

    def _sweep_layer_by_layer(self):
        """Serial baseline (Section 4.1): one pass over the layers, W_l then Z_l, newest values everywhere."""
        L, M = self.L, self.M
        W, Z, U = list(self.W), list(self.Z), self.U
        T_seen = None
        for l in range(1, L + 1):
            W[l] = self.update_W(l, W, Z, U)
            self._trace("W", l, W, Z, U)
            p_prev = self.first_order(l - 1, Z[l - 1], W[l])
            Znew = np.empty_like(Z[l])
            if l < L:
                p_cur = self.first_order(l, Z[l], W[l + 1])
                s_cur = self.second_order(l, p_cur, Z[l + 1], U)
                for m in range(M):
                    Znew[self.g.rows(m)] = self.update_Z_hidden(l, m, Z, W, U, p_prev, p_cur, s_cur)
            else:
                T_seen = np.vstack([sum(p_prev[(r, m)] for r in self.g.nbr_and_self(m)) for m in range(M)])
                for m in range(M):
                    Znew[self.g.rows(m)] = self.update_Z_last(m, Z, U, p_prev)
            Z_L_old = Z[L]
            Z[l] = Znew
            self._trace("Z", l, W, Z, U)
        if self.dual_form == 0:
            Un = U + self.rho * (Z_L_old - T_seen)
        else:
            Un = U + self.rho * (Z[L] - T_seen)     # Z_{L-1}, W_L did not change after the last-layer update
        self.TL_prev = np.vstack([self.g.aggregate_block(m, self.Z[L - 1]) @ self.W[L] for m in range(M)])
        self.W, self.Z, self.U = W, Z, Un
        self.k += 1
        if not all(np.all(np.isfinite(a)) for a in self.W[1:] + self.Z[1:] + [self.U]):
            self.status |= self.STATUS_NONFINITE

    def _trace(self, name, l, W, Z, U):
        if self.block_trace is not None:
            self.block_trace.append((name, l, self.stats_full_graph(W, Z, U)["lagrangian"]))

    def _sweep(self):
        L, M = self.L, self.M
        Wk, Zk, Uk = self.W, self.Z, self.U
        # Algorithm 1, the W step: W_l^{k+1} for every l from (Z^k, U^k)
        Wn = [None] + [self.update_W(l, Wk, Zk, Uk) for l in range(1, L + 1)]
        # messages with Z^k and W^{k+1}
        p = [self.first_order(l, Zk[l], Wn[l + 1]) for l in range(0, L)]
        s = [None] + [self.second_order(l, p[l], Zk[l + 1], Uk) for l in range(1, L)]
        # Algorithm 1, the Z step: Z_{l,m}^{k+1} for every l, m from (W^{k+1}, Z^k, U^k)
        Zn = [Zk[0]] + [np.empty_like(Zk[l]) for l in range(1, L + 1)]
        for l in range(1, L):
            for m in range(M):
                Zn[l][self.g.rows(m)] = self.update_Z_hidden(l, m, Zk, Wn, Uk, p[l - 1], p[l], s[l])
        for m in range(M):
            Zn[L][self.g.rows(m)] = self.update_Z_last(m, Zk, Uk, p[L - 1])
        # Algorithm 1, the dual step: U_m^{k+1} = U_m^k + rho (Z_{L,m}^k - sum_r p_{L-1,r->m}^k)   (Eq. 2 as printed)
        # dual_form 1 is the usual ADMM dual ascent on the new iterates instead:
        #         U_m^{k+1} = U_m^k + rho (Z_{L,m}^{k+1} - sum_r A~_{m,r} Z_{L-1,r}^{k+1} W_L^{k+1})
        Un = np.empty_like(Uk)
        for m in range(M):
            if self.dual_form == 0:
                c = sum(p[L - 1][(r, m)] for r in self.g.nbr_and_self(m))
                Un[self.g.rows(m)] = self.blk(Uk, m) + self.rho * (self.blk(Zk[L], m) - c)
            else:
                c = self.g.aggregate_block(m, Zn[L - 1]) @ Wn[L]
                Un[self.g.rows(m)] = self.blk(Uk, m) + self.rho * (self.blk(Zn[L], m) - c)
        # keep A~ Z_{L-1}^k W_L^k for the dual residual of the next readout
        self.TL_prev = np.vstack([self.g.aggregate_block(m, Zk[L - 1]) @ Wk[L] for m in range(M)])
        self.W, self.Z, self.U = Wn, Zn, Un
        self.k += 1
        if not all(np.all(np.isfinite(a)) for a in self.W[1:] + self.Z[1:] + [self.U]):
            self.status |= self.STATUS_NONFINITE

    # ------------------------------------------------------------------ readout
    def stats(self):
        """Objective of Problem 3, augmented Lagrangian (Eq. 1), residuals, at the current iterate."""
        L, M = self.L, self.M
        risk = sum(self.risk_value(self.blk(self.Z[L], m), self.Y[self.g.rows(m)],
                                   self.labelled[self.g.rows(m)]) for m in range(M))
        pen = [self.phi(l, self.W[l], self.Z[l - 1], self.Z[l]) for l in range(1, L)]
        phiL = self.phi(L, self.W[L], self.Z[L - 1], self.Z[L], self.U)
        TL = np.vstack([self.g.aggregate_block(m, self.Z[L - 1]) @ self.W[L] for m in range(M)])
        primal = float(np.sqrt(sqnorm(self.Z[L] - TL)))
        dual = 0.0 if self.TL_prev is None else self.rho * float(np.sqrt(sqnorm(TL - self.TL_prev)))
        F = risk + sum(pen)
        return dict(objective=F, lagrangian=F + phiL, risk=risk, primal_res=primal, dual_res=dual,
                    layer_penalty=pen, iter=self.k, status=self.status)

    def phi_full_graph(self, l, Wl, Zprev, Zl, U=None):
        """phi in its full-graph form (the right-hand sides of its two definitions in Section 3)."""
        A = self.g.A
        if Wl.shape[0] > Wl.shape[1]:
            T = A @ (Zprev @ Wl)
        elif Zprev is self.Z[0]:                      # A~ Z_0 never changes: keep it between calls
            if getattr(self, "_AZ0", None) is None:
                self._AZ0 = A @ Zprev
            T = self._AZ0 @ Wl
        else:
            T = (A @ Zprev) @ Wl
        if l < self.L:
            return 0.5 * self.nu * sqnorm(Zl - relu(T))
        r = Zl - T
        return inner(U, r) + 0.5 * self.rho * sqnorm(r)

    def stats_full_graph(self, W=None, Z=None, U=None):
        """The same readout from the full-graph forms (right-hand sides of the definitions of phi and of
        Problem 2 / Eq. 1), with the sparse A~ applied to narrow products.  Needs no block split, so it
        runs on graphs with millions of nodes."""
        W = self.W if W is None else W
        Z = self.Z if Z is None else Z
        U = self.U if U is None else U
        L, A = self.L, self.g.A
        risk = self.risk_value(Z[L], self.Y, self.labelled)
        pen = [self.phi_full_graph(l, W[l], Z[l - 1], Z[l]) for l in range(1, L)]
        TL = A @ (Z[L - 1] @ W[L])
        r = Z[L] - TL
        phiL = inner(U, r) + 0.5 * self.rho * sqnorm(r)
        F = risk + sum(pen)
        return dict(objective=F, lagrangian=F + phiL, risk=risk, primal_res=float(np.sqrt(sqnorm(r))),
                    layer_penalty=pen, TL=TL)

    def predict(self):
        """Inference with the current weights (Section 4.2): forward pass of Problem 1's constraints from
        Z_0, class = index of the largest logit.  Returns (classes, logits, accuracy over labelled nodes),
        classes and logits in the caller's node order."""
        Z = self.Z[0]
        for l in range(1, self.L + 1):
            T = np.vstack([self.g.aggregate_block(m, Z) @ self.W[l] for m in range(self.M)])
            Z = relu(T) if l < self.L else T
        pred = np.argmax(Z, axis=1)
        lab = self.labelled
        acc = float(np.mean(pred[lab] == self.labels[lab])) if lab.any() else 0.0
        return self.g.to_old(pred), self.g.to_old(Z), acc

    # ------------------------------------------------------------------ snapshot / restore (tests)
    def snapshot(self):
        return dict(W=[None] + [w.copy() for w in self.W[1:]], Z=[z.copy() for z in self.Z], U=self.U.copy(),
                    tau=list(self.tau), theta=[None] + [list(t) for t in self.theta[1:]], k=self.k,
                    status=self.status, TL_prev=None if self.TL_prev is None else self.TL_prev.copy(),
                    trials_W=list(self.trials_W), trials_Z=[None] + [list(t) for t in self.trials_Z[1:]])

    def restore(self, snap):
        snap = dict(snap)
        self.W = [None] + [w.copy() for w in snap["W"][1:]]
        self.Z = [z.copy() for z in snap["Z"]]
        self.U = snap["U"].copy()
        self.tau = list(snap["tau"])
        self.theta = [None] + [list(t) for t in snap["theta"][1:]]
        self.k, self.status = snap["k"], snap["status"]
        self.TL_prev = None if snap["TL_prev"] is None else snap["TL_prev"].copy()
        self.trials_W = list(snap["trials_W"])
        self.trials_Z = [None] + [list(t) for t in snap["trials_Z"][1:]]

    # ------------------------------------------------------------------ accessors (caller's node order)
    def get_W(self, l):
        return self.W[l].copy()

    def get_Z(self, l):
        return self.g.to_old(self.Z[l])

    def get_U(self):
        return self.g.to_old(self.U)

    def get_steps(self):
        tau = np.array(self.tau[1:], dtype=np.float64)
        theta = np.array([self.theta[l][m] for l in range(1, self.L) for m in range(self.M)], dtype=np.float64)
        trials = np.array(self.trials_W[1:] + [self.trials_Z[l][m] for l in range(1, self.L)
                                                for m in range(self.M)], dtype=np.int32)
        return tau, theta, trials


def make_oracle(w, iters=None):
    """Build graph + oracle for a synth.Workload-like object (attributes only, no import of the generator)."""
    g = OracleGraph(w.N, w.src, w.dst, w.M, w.comm)
    h = w.hyper
    o = AdmmOracle(g, w.dims, nu=h["nu"], rho=h["rho"], tau0=h["tau0"], theta0=h["theta0"], eta=h["eta"],
                   max_backtrack=h["max_backtrack"], fista_iters=h["fista_iters"], risk=h["risk"],
                   dual_form=h["dual_form"], schedule=h.get("schedule", 0), step_policy=h.get("step_policy", 0),
                   fista_mode=h.get("fista_mode", 0))
    o.set_data(w.X, w.labels)
    o.init(w.W0)
    return o
