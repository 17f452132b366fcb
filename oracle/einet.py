"""Float64 NumPy oracle of the EiNet forward pass and EM (test infrastructure).

Written from the definitions in the paper, node by node, with none of the
blocking, fusion or linear-domain tricks of the GPU path:

* leaves      : exponential-family log-density  log h(x) + T(x).theta - A(theta)
                with expectation parameters phi (Sec. 3.4); a leaf region is
                the factorisation (sum of logs) over its scope; a marginalised
                variable contributes log 1 = 0 (Sec. 2, decomposability);
* partition   : log S_k = logsumexp_ij( log W_kij + log N_i + log N'_j ), the
                plain log-domain form of Eq. 3 (the prior-art way of Sec. 3.2,
                not the shifted linear-domain form of Eq. 4);
* region with several partitions: element-wise mixture of its simple sums
                (App. B), log S_k = logsumexp_c( log v_kc + log S^c_k );
* E-step      : n = w * dlogP/dw and p = dlogP/dlogL (Eq. 6 and the two
                derivations after Eq. 7), obtained by the explicit top-down
                recursion of the latent-variable posterior;
* M-step      : Eq. 7, then the stochastic-EM blend of Eq. 8-9 and the
                variance projection of Sec. 4.2.

Readings of points the paper leaves open (same on the GPU side, by
specification, not by shared code):
  - the root region has a single entry (K_out = 1);
  - mixing weights are private per entry k: v[s][k][c], sum_c v = 1;
  - EM with marginalised variables is exact EM for missing data: a masked
    (sample, variable) pair contributes the leaf's current expectation,
    phi_hat = (num + (tot - den) * phi_old) / tot, which is Eq. 7 when nothing
    is masked;
  - a weight row or a leaf entry with zero accumulated posterior keeps its
    old value; weights are floored at w_floor and renormalised before the
    blend; the variance projection is applied after the blend.
"""
from __future__ import annotations

import numpy as np

from .structure import RegionGraph, param_layout

BERNOULLI = 0
GAUSSIAN = 1
BINOMIAL = 2      # leaf_param = number of trials N; x in {0..N}; phi = E[x] = N p
CATEGORICAL = 3   # leaf_param = number of values V; x in {0..V-1}; phi = the V probabilities
NUM_STATS = {BERNOULLI: 1, GAUSSIAN: 2}
P_MIN = 1e-6  # probabilities are kept in [P_MIN, 1 - P_MIN] (categorical: >= P_MIN, renormalised) by the M-step


def num_stats(family, leaf_param=0):
    """|T|, the dimension of the sufficient statistic (Sec. 3.4)."""
    if family == CATEGORICAL:
        return int(leaf_param)
    return 1 if family in (BERNOULLI, BINOMIAL) else 2


def _logsumexp(a, axis):
    m = np.max(a, axis=axis, keepdims=True)
    m = np.where(np.isfinite(m), m, 0.0)
    with np.errstate(divide="ignore"):
        out = np.log(np.sum(np.exp(a - m), axis=axis, keepdims=True)) + m
    return np.squeeze(out, axis=axis)


def ef_log_density(family, x, phi, leaf_param=0):
    """log h(x) + T(x).theta(phi) - A(theta)  (Sec. 3.4).

    x   : [...]        values
    phi : [T, ...]     expectation parameters, broadcastable against x
    leaf_param : trials N (binomial) or number of values V (categorical)
    """
    if family == BINOMIAL:
        from scipy.special import gammaln
        N = float(leaf_param)
        p = phi[0] / N                          # phi = E[x] = N p
        theta = np.log(p) - np.log1p(-p)
        A = -N * np.log1p(-p)
        log_h = gammaln(N + 1.0) - gammaln(x + 1.0) - gammaln(N - x + 1.0)      # log of the binomial coefficient
        return log_h + x * theta - A
    if family == CATEGORICAL:
        # T(x) = indicator vector of the value, theta_v = log phi_v, h = 1, A = 0 on the simplex
        Tx = suff_stats(CATEGORICAL, x, leaf_param)
        with np.errstate(divide="ignore"):
            theta = np.log(phi)
        out = 0.0
        for v in range(int(leaf_param)):
            out = out + np.where(Tx[v] != 0, theta[v], 0.0)
        return out
    if family == BERNOULLI:
        # h(x) = 1, T(x) = x, theta = log p - log(1-p), A = -log(1-p):  x theta - A = x log p + (1-x) log(1-p).
        # Written in the second form so that the boundary of the parameter space (p = 0 or 1, where theta is
        # infinite) gives the density p^x (1-p)^(1-x) itself: an exponent of 0 contributes log 1 = 0.
        p = phi[0] + 0.0 * x
        xx = x + 0.0 * p
        with np.errstate(divide="ignore", invalid="ignore"):
            a = np.where(xx != 0, xx * np.log(p), 0.0)
            b = np.where(xx != 1, (1.0 - xx) * np.log1p(-p), 0.0)
        return a + b
    if family == GAUSSIAN:
        mu = phi[0]
        var = phi[1] - phi[0] ** 2              # phi = (E[x], E[x^2])
        theta1 = mu / var
        theta2 = -0.5 / var
        A = mu ** 2 / (2.0 * var) + 0.5 * np.log(var)
        log_h = -0.5 * np.log(2.0 * np.pi)
        return log_h + x * theta1 + x * x * theta2 - A
    raise ValueError("unknown leaf family")


def suff_stats(family, x, leaf_param=0):
    """T(x) stacked on a new leading axis."""
    if family in (BERNOULLI, BINOMIAL):
        return np.stack([x])
    if family == CATEGORICAL:
        return np.stack([(x == v).astype(np.float64) for v in range(int(leaf_param))])
    return np.stack([x, x * x])


class OracleEiNet:
    def __init__(self, graph: RegionGraph, K: int, channels: int, family: int, leaf_param: int = 0):
        self.g = graph
        self.K = K
        self.C = channels
        self.family = family
        self.leaf_param = leaf_param
        self.T = num_stats(family, leaf_param)
        self.layout = param_layout(graph, K, channels, self.T)
        self.W = [None] * graph.num_partitions        # [K_out, K, K]
        self.v = {}                                   # region -> [K_out, C_s]
        self.phi = None                               # [D, C, R, T, K]
        # children-before-parents order by depth-first search from the root
        self._post = []
        seen = set()

        def visit(s):
            if s in seen:
                return
            seen.add(s)
            for n in graph.children[s]:
                _, left, right = graph.partitions[n]
                visit(left)
                visit(right)
            self._post.append(s)

        import sys
        old = sys.getrecursionlimit()
        sys.setrecursionlimit(max(old, 10000))
        try:
            visit(0)
        finally:
            sys.setrecursionlimit(old)

    # ---------------------------------------------------------------- params
    def set_flat_params(self, flat):
        flat = np.asarray(flat, dtype=np.float64)
        g, K, lay = self.g, self.K, self.layout
        assert flat.size == lay.n_params
        for n, (parent, _, _) in enumerate(g.partitions):
            ko = g.k_out(parent, K)
            self.W[n] = flat[lay.w_off[n]: lay.w_off[n] + ko * K * K].reshape(ko, K, K).copy()
        self.v = {}
        for s, off in lay.v_off.items():
            ko, c = g.k_out(s, K), len(g.children[s])
            self.v[s] = flat[off: off + ko * c].reshape(ko, c).copy()
        self.phi = flat[lay.phi_off:].reshape(g.num_vars, self.C, g.num_replica, self.T, K).copy()

    def get_flat_params(self):
        parts = [w.ravel() for w in self.W]
        parts += [self.v[s].ravel() for s in sorted(self.v)]
        parts.append(self.phi.ravel())
        return np.concatenate(parts)

    @staticmethod
    def _mask(mask, B, D):
        if mask is None:
            return np.ones((B, D))
        m = np.asarray(mask, dtype=np.float64)
        if m.ndim == 1:
            m = np.broadcast_to(m[None, :], (B, D))
        assert m.shape == (B, D)
        return m

    # --------------------------------------------------------------- forward
    def forward(self, x, mask=None):
        """Returns (logp[B], N, S): N[region] -> [B, K_out] log-densities,
        S[partition] -> [B, K_out] log-values of the simple sums."""
        g, K = self.g, self.K
        x = np.asarray(x, dtype=np.float64)
        B = x.shape[0]
        assert x.shape == (B, g.num_vars, self.C)
        m = self._mask(mask, B, g.num_vars)
        N, S = {}, {}
        with np.errstate(divide="ignore"):
            logW = [np.log(w) for w in self.W]
            logv = {s: np.log(v) for s, v in self.v.items()}
        for s in self._post:
            if g.is_leaf(s):
                r = g.replica[s]
                acc = np.zeros((B, K))
                for d in g.scopes[s]:
                    for c in range(self.C):
                        e = ef_log_density(self.family, x[:, d, c][:, None],
                                           self.phi[d, c, r][:, None, :], self.leaf_param)      # [B, K]
                        acc += np.where(m[:, d][:, None] != 0, e, 0.0)      # marginalised: factor 1, whatever e is
                N[s] = acc
                continue
            simple = []
            for n in g.children[s]:
                _, left, right = g.partitions[n]
                a = (logW[n][None, :, :, :]
                     + N[left][:, None, :, None]
                     + N[right][:, None, None, :])                             # [B, K_out, K, K]
                S[n] = _logsumexp(a.reshape(B, a.shape[1], K * K), axis=2)
                simple.append(S[n])
            if len(simple) == 1:
                N[s] = simple[0]
            else:
                stack = np.stack(simple, axis=2) + logv[s][None, :, :]           # [B, K_out, C_s]
                N[s] = _logsumexp(stack, axis=2)
        return N[0][:, 0].copy(), N, S

    def logp(self, x, mask=None, chunk=None):
        x = np.asarray(x, dtype=np.float64)
        B = x.shape[0]
        if chunk is None or chunk >= B:
            return self.forward(x, mask)[0]
        m = None if mask is None else np.asarray(mask)
        out = []
        for b0 in range(0, B, chunk):
            mm = m if (m is None or m.ndim == 1) else m[b0:b0 + chunk]
            out.append(self.forward(x[b0:b0 + chunk], mm)[0])
        return np.concatenate(out)

    def conditional_logp(self, x, query, evidence):
        """log p(x_q | x_e) of Eq. 1: ratio of two marginals; variables in
        neither set are integrated out in both."""
        q = np.asarray(query, dtype=np.float64)
        e = np.asarray(evidence, dtype=np.float64)
        assert not np.any((q > 0) & (e > 0))
        return self.logp(x, np.maximum(q, e)) - self.logp(x, e)

    # ---------------------------------------------------------------- E-step
    def zero_stats(self):
        g, K = self.g, self.K
        return {
            "Nw": [np.zeros_like(w) for w in self.W],
            "Nv": {s: np.zeros_like(v) for s, v in self.v.items()},
            "num": np.zeros_like(self.phi),
            "den": np.zeros((g.num_vars, g.num_replica, K)),
            "tot": np.zeros((g.num_vars, g.num_replica, K)),
        }

    def em_accumulate(self, x, mask=None, stats=None, chunk=None, want_grads=False):
        """Adds the expected statistics of the batch (Eq. 6) to ``stats``.
        Returns (stats, logp[B]) (and the per-region posteriors G if asked)."""
        x = np.asarray(x, dtype=np.float64)
        B = x.shape[0]
        if stats is None:
            stats = self.zero_stats()
        if chunk is not None and chunk < B and not want_grads:
            m = None if mask is None else np.asarray(mask)
            lps = []
            for b0 in range(0, B, chunk):
                mm = m if (m is None or m.ndim == 1) else m[b0:b0 + chunk]
                _, lp = self.em_accumulate(x[b0:b0 + chunk], mm, stats)
                lps.append(lp)
            return stats, np.concatenate(lps)

        g, K = self.g, self.K
        m = self._mask(mask, B, g.num_vars)
        logp, N, S = self.forward(x, mask)
        with np.errstate(divide="ignore"):
            logW = [np.log(w) for w in self.W]
            logv = {s: np.log(v) for s, v in self.v.items()}
        G = {s: np.zeros((B, g.k_out(s, K))) for s in range(g.num_regions)}
        G[0][:] = 1.0                                    # dlogP/dlogP
        for s in reversed(self._post):                   # parents before children
            Gs = G[s]
            if g.is_leaf(s):
                r = g.replica[s]
                for d in g.scopes[s]:
                    stats["tot"][d, r] += Gs.sum(0)
                    stats["den"][d, r] += (m[:, d][:, None] * Gs).sum(0)
                    for c in range(self.C):
                        Tx = suff_stats(self.family, x[:, d, c], self.leaf_param)            # [T, B]
                        stats["num"][d, c, r] += np.einsum("tb,b,bk->tk", Tx, m[:, d], Gs)
                continue
            ch = g.children[s]
            for ci, n in enumerate(ch):
                _, left, right = g.partitions[n]
                if len(ch) > 1:
                    rho = np.exp(logv[s][None, :, ci] + S[n] - N[s])            # [B, K_out]
                    Gn = Gs * rho
                    stats["Nv"][s][:, ci] += Gn.sum(0)
                else:
                    Gn = Gs
                V = Gn[:, :, None, None] * np.exp(
                    logW[n][None, :, :, :]
                    + N[left][:, None, :, None]
                    + N[right][:, None, None, :]
                    - S[n][:, :, None, None])                                   # [B, K_out, K, K]
                stats["Nw"][n] += V.sum(0)
                G[left] += V.sum(axis=(1, 3))
                G[right] += V.sum(axis=(1, 2))
        if want_grads:
            return stats, logp, G
        return stats, logp

    # ---------------------------------------------------------------- M-step
    def em_update(self, stats, step=1.0, min_var=0.0, max_var=np.inf, w_floor=0.0):
        """Eq. 7 on the accumulated statistics, blended with step size
        lambda = step (Eq. 8-9), variance projected to [min_var, max_var]
        afterwards (Sec. 4.2).  Updates the parameters in place."""
        lam = float(step)

        def new_weights(old, n_acc):
            # rows: last axes flattened are the children of one sum entry
            shp = old.shape
            o = old.reshape(shp[0], -1)
            a = n_acc.reshape(shp[0], -1)
            tot = a.sum(axis=1, keepdims=True)
            with np.errstate(invalid="ignore", divide="ignore"):
                hat = np.where(tot > 0, a / tot, o)
            if w_floor > 0:
                hat = np.maximum(hat, w_floor)
                hat = hat / hat.sum(axis=1, keepdims=True)
            return ((1.0 - lam) * o + lam * hat).reshape(shp)

        for n in range(len(self.W)):
            self.W[n] = new_weights(self.W[n], stats["Nw"][n])
        for s in self.v:
            self.v[s] = new_weights(self.v[s], stats["Nv"][s])

        tot = stats["tot"][:, None, :, None, :]          # [D,1,R,1,K]
        den = stats["den"][:, None, :, None, :]
        with np.errstate(invalid="ignore", divide="ignore"):
            hat = np.where(tot > 0, (stats["num"] + (tot - den) * self.phi) / tot, self.phi)
        phi = (1.0 - lam) * self.phi + lam * hat
        if self.family == BERNOULLI:
            phi = np.clip(phi, P_MIN, 1.0 - P_MIN)
        elif self.family == BINOMIAL:
            phi = np.clip(phi, self.leaf_param * P_MIN, self.leaf_param * (1.0 - P_MIN))
        elif self.family == CATEGORICAL:
            phi = np.maximum(phi, P_MIN)
            phi = phi / phi.sum(axis=3, keepdims=True)
        else:
            mu = phi[:, :, :, 0, :]
            var = np.clip(phi[:, :, :, 1, :] - mu ** 2, min_var, max_var)
            phi[:, :, :, 1, :] = mu ** 2 + var
        self.phi = phi

    def stats_to_flat(self, stats):
        parts = [a.ravel() for a in stats["Nw"]]
        parts += [stats["Nv"][s].ravel() for s in sorted(stats["Nv"])]
        parts += [stats["num"].ravel(), stats["den"].ravel(), stats["tot"].ravel()]
        return np.concatenate(parts)

    def stats_from_flat(self, flat):
        """Inverse of stats_to_flat."""
        flat = np.asarray(flat, dtype=np.float64)
        lay, st = self.layout, self.zero_stats()
        assert flat.size == lay.n_stats
        for n, w in enumerate(self.W):
            st["Nw"][n] = flat[lay.w_off[n]: lay.w_off[n] + w.size].reshape(w.shape).copy()
        for s, v in self.v.items():
            st["Nv"][s] = flat[lay.v_off[s]: lay.v_off[s] + v.size].reshape(v.shape).copy()
        st["num"] = flat[lay.phi_off: lay.n_params].reshape(self.phi.shape).copy()
        st["den"] = flat[lay.den_off: lay.tot_off].reshape(st["den"].shape).copy()
        st["tot"] = flat[lay.tot_off:].reshape(st["tot"].shape).copy()
        return st
