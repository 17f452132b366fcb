"""Pins for the float64 oracle: every check compares it with something that is
not the oracle itself: brute-force enumeration, library routines on special
cases that reduce to textbook models, closed forms, finite differences and the
invariants the paper states for smooth, decomposable circuits."""
import numpy as np
import pytest
import scipy.special
import scipy.stats

from oracle import structure as S
from oracle.einet import OracleEiNet, BERNOULLI, GAUSSIAN, ef_log_density
from tests.common import normalise_exactly, make_oracle, make_config, all_binary


RAT_TINY = dict(kind="rat", D=8, depth=3, R=2)


# ----------------------------------------------------------------------------- leaves
def test_leaf_families_match_scipy():
    rng = np.random.default_rng(0)
    x = rng.normal(size=50)
    mu, var = rng.normal(size=50), rng.uniform(1e-6, 3.0, size=50)
    got = ef_log_density(GAUSSIAN, x, np.stack([mu, mu ** 2 + var]))
    np.testing.assert_allclose(got, scipy.stats.norm.logpdf(x, mu, np.sqrt(var)), rtol=1e-9, atol=1e-6)
    xb = (rng.random(50) < 0.5).astype(float)
    p = rng.uniform(0.01, 0.99, size=50)
    got = ef_log_density(BERNOULLI, xb, np.stack([p]))
    np.testing.assert_allclose(got, scipy.stats.bernoulli.logpmf(xb, p), rtol=1e-12)


# ----------------------------------------------------------------------------- P1 normalisation
@pytest.mark.parametrize("spec,K", [
    (RAT_TINY, 4),                                         # configuration 1 of the benchmark
    (dict(kind="rat", D=11, depth=2, R=3), 3),
    (dict(kind="pd", H=3, W=3, deltas=[1]), 3),            # regions shared between parents
    (dict(kind="pd", H=2, W=6, deltas=[2, 1]), 2),
])
def test_sums_to_one_over_all_binary_states(spec, K):
    model, _, _ = make_oracle(spec, K, 1, BERNOULLI, seed=5)
    normalise_exactly(model)
    X = all_binary(model.g.num_vars)
    logp = model.logp(X)
    assert abs(np.exp(logp).sum() - 1.0) < 1e-12
    # every inner region is a normalised density over its own scope as well (Sec. 2, smoothness)
    _, N, _ = model.forward(X)
    for s in (1, model.g.num_regions // 2):
        scope = list(model.g.scopes[s])
        # sum over the states of the scope, any fixed completion outside it
        states = [i for i in range(len(X)) if all(X[i, d, 0] == 0 for d in range(model.g.num_vars) if d not in scope)]
        tot = np.exp(N[s][states]).sum(axis=0)
        np.testing.assert_allclose(tot, 1.0, atol=1e-12)


def test_config1_normalisation_with_float32_parameters():
    cfg, model, flat, x, mask = make_config(1)
    logp = model.logp(all_binary(8))
    assert abs(np.exp(logp).sum() - 1.0) < 1e-5           # rows are float32-rounded Dirichlet draws
    assert x.shape == (64, 8, 1) and set(np.unique(x)) <= {0.0, 1.0}


# ----------------------------------------------------------------------------- P2 marginals, Eq. 1
@pytest.mark.parametrize("family", [BERNOULLI, GAUSSIAN])
def test_everything_marginalised_gives_zero(family):
    model, _, rng = make_oracle(dict(kind="pd", H=4, W=4, deltas=[2]), 3, 2, family, seed=1)
    normalise_exactly(model)
    x = rng.random((5, 16, 2))
    assert np.max(np.abs(model.logp(x, np.zeros(16)))) < 1e-13
    assert np.max(np.abs(model.logp(x, np.zeros((5, 16))))) < 1e-13


def test_marginal_consistency_and_conditionals():
    model, _, rng = make_oracle(RAT_TINY, 4, 1, BERNOULLI, seed=2)
    normalise_exactly(model)
    D = 8
    e = np.array([1, 0, 0, 1, 0, 0, 1, 0])       # evidence
    q = np.array([0, 1, 0, 0, 1, 0, 0, 0])       # query; variables 2, 5, 7 are missing
    x = (rng.random((1, D, 1)) < 0.5).astype(float)
    p_e = np.exp(model.logp(x, e))[0]
    tot_joint, tot_cond = 0.0, 0.0
    for a in (0.0, 1.0):
        for b in (0.0, 1.0):
            xx = x.copy(); xx[0, 1, 0] = a; xx[0, 4, 0] = b
            tot_joint += np.exp(model.logp(xx, np.maximum(q, e)))[0]
            tot_cond += np.exp(model.conditional_logp(xx, q, e))[0]
    assert abs(tot_joint - p_e) < 1e-14                   # sum_q P(x_q, x_e) = P(x_e)
    assert abs(tot_cond - 1.0) < 1e-12                    # Eq. 1 is a distribution over x_q
    # Eq. 1 against the definition by explicit summation over the missing variables
    full = all_binary(D)
    lp = model.logp(full)
    sel_e = np.all(full[:, e == 1, 0] == x[0, e == 1, 0], axis=1)
    sel_q = sel_e & np.all(full[:, q == 1, 0] == x[0, q == 1, 0], axis=1)
    want = np.log(np.exp(lp[sel_q]).sum() / np.exp(lp[sel_e]).sum())
    assert abs(model.conditional_logp(x, q, e)[0] - want) < 1e-12
    # per-sample masks behave like per-row shared masks
    xs = (rng.random((3, D, 1)) < 0.5).astype(float)
    ms = (rng.random((3, D)) < 0.5).astype(float)
    rows = [model.logp(xs[i:i + 1], ms[i])[0] for i in range(3)]
    np.testing.assert_allclose(model.logp(xs, ms), rows, rtol=0, atol=1e-14)


# ----------------------------------------------------------------------------- P3 special cases
@pytest.mark.parametrize("family", [BERNOULLI, GAUSSIAN])
def test_k1_r1_is_a_fully_factorised_model(family):
    model, _, rng = make_oracle(dict(kind="rat", D=9, depth=2, R=1), 1, 2, family, seed=3)
    B, D, C = 40, 9, 2
    if family == BERNOULLI:
        x = (rng.random((B, D, C)) < 0.3).astype(float)
        p = model.phi[:, :, 0, 0, 0]
        want = scipy.stats.bernoulli.logpmf(x, p[None]).sum(axis=(1, 2))
    else:
        x = rng.normal(0.3, 2.0, size=(B, D, C))
        mu = model.phi[:, :, 0, 0, 0]
        sd = np.sqrt(model.phi[:, :, 0, 1, 0] - mu ** 2)
        want = scipy.stats.norm.logpdf(x, mu[None], sd[None]).sum(axis=(1, 2))
    np.testing.assert_allclose(model.logp(x), want, rtol=1e-12)
    # one full EM step is the maximum-likelihood fit: sample mean and (biased) sample variance
    stats, _ = model.em_accumulate(x)
    model.em_update(stats, step=1.0)
    np.testing.assert_allclose(model.phi[:, :, 0, 0, 0], x.mean(axis=0), rtol=1e-12)
    if family == GAUSSIAN:
        var = model.phi[:, :, 0, 1, 0] - model.phi[:, :, 0, 0, 0] ** 2
        np.testing.assert_allclose(var, x.var(axis=0), rtol=1e-9)
    assert all(np.all(w == 1.0) for w in model.W)


def test_depth1_is_a_mixture_with_k_squared_components():
    K = 3
    model, _, rng = make_oracle(dict(kind="rat", D=7, depth=1, R=1), K, 1, GAUSSIAN, seed=4)
    g = model.g
    x = rng.normal(0.5, 1.0, size=(20, 7, 1))
    mu = model.phi[:, 0, 0, 0, :]
    sd = np.sqrt(model.phi[:, 0, 0, 1, :] - mu ** 2)
    lp = scipy.stats.norm.logpdf(x[:, :, 0, None], mu[None], sd[None])          # [B, D, K]
    left = lp[:, list(g.scopes[1]), :].sum(axis=1)                               # [B, K]
    right = lp[:, list(g.scopes[2]), :].sum(axis=1)
    comp = np.log(model.W[0][0])[None] + left[:, :, None] + right[:, None, :]    # [B, K, K]
    want = scipy.special.logsumexp(comp.reshape(20, -1), axis=1)
    np.testing.assert_allclose(model.logp(x), want, rtol=1e-12)
    # transposing W must change the answer (left/right are not interchangeable)
    model.W[0] = model.W[0].transpose(0, 2, 1).copy()
    assert np.max(np.abs(model.logp(x) - want)) > 1e-3


def test_k1_replicas_are_a_textbook_mixture_and_em_matches():
    R, D, B = 4, 6, 200
    model, _, rng = make_oracle(dict(kind="rat", D=D, depth=2, R=R), 1, 1, BERNOULLI, seed=6)
    normalise_exactly(model)
    x = (rng.random((B, D, 1)) < rng.uniform(0.2, 0.8, size=(1, D, 1))).astype(float)
    pi = model.v[0][0].copy()                        # root mixing weights
    p = model.phi[:, 0, :, 0, 0].copy()              # [D, R]
    comp = np.log(pi)[None] + scipy.stats.bernoulli.logpmf(x[:, :, 0, None], p[None]).sum(axis=1)   # [B, R]
    np.testing.assert_allclose(model.logp(x), scipy.special.logsumexp(comp, axis=1), rtol=1e-12)
    resp = scipy.special.softmax(comp, axis=1)
    stats, _ = model.em_accumulate(x)
    np.testing.assert_allclose(stats["Nv"][0][0], resp.sum(axis=0), rtol=1e-12)
    model.em_update(stats, step=1.0)
    np.testing.assert_allclose(model.v[0][0], resp.mean(axis=0), rtol=1e-12)
    want_p = np.einsum("br,bd->dr", resp, x[:, :, 0]) / resp.sum(axis=0)[None]
    np.testing.assert_allclose(model.phi[:, 0, :, 0, 0], np.clip(want_p, 1e-6, 1 - 1e-6), rtol=1e-12)
    # stochastic EM (Eq. 8-9) is the convex blend of old and new
    model2, _, _ = make_oracle(dict(kind="rat", D=D, depth=2, R=R), 1, 1, BERNOULLI, seed=6)
    normalise_exactly(model2)
    stats2, _ = model2.em_accumulate(x)
    model2.em_update(stats2, step=0.25)
    np.testing.assert_allclose(model2.v[0][0], 0.75 * pi + 0.25 * resp.mean(axis=0), rtol=1e-12)
    np.testing.assert_allclose(model2.phi[:, 0, :, 0, 0], 0.75 * p + 0.25 * want_p, rtol=1e-12)


# ----------------------------------------------------------------------------- P4 Eq. 2 / Eq. 5
def test_partition_is_the_linear_domain_einsum():
    model, _, rng = make_oracle(RAT_TINY, 4, 1, BERNOULLI, seed=7)
    x = (rng.random((10, 8, 1)) < 0.5).astype(float)
    _, N, Sv = model.forward(x)
    for n, (parent, left, right) in enumerate(model.g.partitions):
        lin = np.einsum("kij,bi,bj->bk", model.W[n], np.exp(N[left]), np.exp(N[right]))
        np.testing.assert_allclose(np.exp(Sv[n]), lin, rtol=1e-12)
    # root mixing (App. B): S_k = sum_c v_kc S^c_k
    mix = sum(model.v[0][None, :, c] * np.exp(Sv[n]) for c, n in enumerate(model.g.children[0]))
    np.testing.assert_allclose(np.exp(N[0]), mix, rtol=1e-12)


def test_log_domain_is_stable_far_below_underflow():
    # narrow Gaussians far from the data: densities around exp(-1e6); compare with exact mixture algebra
    K = 2
    model, _, rng = make_oracle(dict(kind="rat", D=4, depth=1, R=1), K, 1, GAUSSIAN, seed=8)
    mu = model.phi[:, :, :, 0, :]
    model.phi[:, :, :, 1, :] = mu ** 2 + 1e-6
    x = rng.uniform(2.0, 3.0, size=(6, 4, 1))
    got = model.logp(x)
    assert np.all(np.isfinite(got)) and np.all(got < -1e5)
    sd = np.sqrt(model.phi[:, 0, 0, 1, :] - model.phi[:, 0, 0, 0, :] ** 2)       # 1e-3 up to rounding of phi
    lp = scipy.stats.norm.logpdf(x[:, :, 0, None], model.phi[:, 0, 0, 0, :][None], sd[None])
    left = lp[:, list(model.g.scopes[1])].sum(axis=1); right = lp[:, list(model.g.scopes[2])].sum(axis=1)
    comp = np.log(model.W[0][0])[None] + left[:, :, None] + right[:, None, :]
    np.testing.assert_allclose(got, scipy.special.logsumexp(comp.reshape(6, -1), axis=1), rtol=1e-10)


# ----------------------------------------------------------------------------- P5 gradients
def test_weight_statistics_are_w_times_gradient():
    """n = w * dlogP/dw (derivation after Eq. 7), by central differences of the forward pass."""
    model, _, rng = make_oracle(dict(kind="pd", H=2, W=4, deltas=[1]), 3, 1, GAUSSIAN, seed=9)
    x = rng.random((7, 8, 1))
    mask = (rng.random((7, 8)) < 0.7).astype(float)
    stats, _ = model.em_accumulate(x, mask)
    eps = 1e-6
    checked = 0
    for n in (0, 3, model.g.num_partitions - 1):
        for idx in [(0, 0, 0), (0, 1, 2), (model.W[n].shape[0] - 1, 2, 1)]:
            w0 = model.W[n][idx]
            model.W[n][idx] = w0 + eps; up = model.logp(x, mask).sum()
            model.W[n][idx] = w0 - eps; dn = model.logp(x, mask).sum()
            model.W[n][idx] = w0
            assert abs(w0 * (up - dn) / (2 * eps) - stats["Nw"][n][idx]) < 1e-7 * max(1.0, stats["Nw"][n][idx])
            checked += 1
    for s in list(model.v)[:3]:
        for idx in [(0, 0), (model.v[s].shape[0] - 1, model.v[s].shape[1] - 1)]:
            v0 = model.v[s][idx]
            model.v[s][idx] = v0 + eps; up = model.logp(x, mask).sum()
            model.v[s][idx] = v0 - eps; dn = model.logp(x, mask).sum()
            model.v[s][idx] = v0
            assert abs(v0 * (up - dn) / (2 * eps) - stats["Nv"][s][idx]) < 1e-7 * max(1.0, stats["Nv"][s][idx])
            checked += 1
    assert checked >= 13


def test_leaf_statistics_are_gradients_wrt_leaf_log_density():
    """p = dlogP/dlogL: perturbing phi moves logP by sum_b p * dlogL/dphi (chain rule)."""
    model, _, rng = make_oracle(dict(kind="rat", D=6, depth=2, R=2), 3, 1, BERNOULLI, seed=10)
    x = (rng.random((9, 6, 1)) < 0.5).astype(float)
    mask = (rng.random((9, 6)) < 0.8).astype(float)
    stats, _ = model.em_accumulate(x, mask)
    eps = 1e-6
    for (d, r, k) in [(0, 0, 0), (3, 1, 2), (5, 0, 1)]:
        p0 = model.phi[d, 0, r, 0, k]
        model.phi[d, 0, r, 0, k] = p0 + eps; up = model.logp(x, mask).sum()
        model.phi[d, 0, r, 0, k] = p0 - eps; dn = model.logp(x, mask).sum()
        model.phi[d, 0, r, 0, k] = p0
        num, den = stats["num"][d, 0, r, 0, k], stats["den"][d, r, k]
        # d/dp [x log p + (1-x) log(1-p)] = x/p - (1-x)/(1-p), weighted by the posterior of the leaf entry
        want = num / p0 - (den - num) / (1 - p0)
        assert abs((up - dn) / (2 * eps) - want) < 1e-6


# ----------------------------------------------------------------------------- P6 invariants
@pytest.mark.parametrize("spec,family,C", [(RAT_TINY, BERNOULLI, 1),
                                           (dict(kind="pd", H=6, W=6, deltas=[2]), GAUSSIAN, 3)])
def test_posterior_bookkeeping(spec, family, C):
    model, _, rng = make_oracle(spec, 3, C, family, seed=12)
    g, B = model.g, 6
    x = rng.random((B, g.num_vars, C))
    if family == BERNOULLI:
        x = (x < 0.5).astype(float)
    stats, logp, G = model.em_accumulate(x, want_grads=True)
    # each variable is explained by exactly one leaf entry per sample
    for d in range(g.num_vars):
        tot = sum(G[s].sum(axis=1) for s in g.leaves() if d in g.scopes[s])
        np.testing.assert_allclose(tot, 1.0, rtol=1e-10)
    # every sum entry that is responsible picks exactly one (i, j): sum_ij Nw = posterior mass that reached it
    np.testing.assert_allclose(sum(stats["Nw"][n].sum() for n in g.children[0]), B, rtol=1e-10)
    for s in model.v:
        np.testing.assert_allclose(stats["Nv"][s].sum(axis=1), G[s].sum(axis=0), rtol=1e-10)
    np.testing.assert_allclose(stats["tot"].sum(axis=(1, 2)), B, rtol=1e-10)
    np.testing.assert_allclose(stats["den"], stats["tot"], rtol=1e-12)       # nothing masked


# ----------------------------------------------------------------------------- P8 brute-force posteriors
def induced_trees(model, s, k):
    """Every way to pick one child at each sum entry reachable from entry k of region s:
    yields (product of the weights picked, list of picks, list of leaf entries reached)."""
    g, K = model.g, model.K
    if g.is_leaf(s):
        yield 1.0, [], [(s, k)]
        return
    ch = g.children[s]
    for ci, n in enumerate(ch):
        wv = model.v[s][k, ci] if len(ch) > 1 else 1.0
        _, left, right = g.partitions[n]
        for i in range(K):
            for j in range(K):
                w = model.W[n][k, i, j]
                for wl, cl, ll in induced_trees(model, left, i):
                    for wr, cr, lr in induced_trees(model, right, j):
                        picks = ([("v", s, k, ci)] if len(ch) > 1 else []) + [("w", n, k, i, j)] + cl + cr
                        yield wv * w * wl * wr, picks, ll + lr


@pytest.mark.parametrize("spec", [dict(kind="rat", D=4, depth=2, R=2), dict(kind="pd", H=1, W=3, deltas=[1])])
def test_em_counts_equal_brute_force_posteriors(spec):
    model, _, rng = make_oracle(spec, 2, 1, BERNOULLI, seed=13)
    normalise_exactly(model)
    g = model.g
    D = g.num_vars
    x = (rng.random((5, D, 1)) < 0.5).astype(float)
    trees = list(induced_trees(model, 0, 0))
    want_w = [np.zeros_like(w) for w in model.W]
    want_v = {s: np.zeros_like(v) for s, v in model.v.items()}
    want_tot = np.zeros((D, g.num_replica, model.K))
    want_num = np.zeros((D, g.num_replica, model.K))
    want_logp = []
    for b in range(len(x)):
        joint = []
        for w, picks, leaves in trees:
            for (s, k) in leaves:
                r = g.replica[s]
                for d in g.scopes[s]:
                    w = w * scipy.stats.bernoulli.pmf(x[b, d, 0], model.phi[d, 0, r, 0, k])
            joint.append(w)
        joint = np.array(joint)
        want_logp.append(np.log(joint.sum()))
        post = joint / joint.sum()
        for pr, (_, picks, leaves) in zip(post, trees):
            for pick in picks:
                if pick[0] == "w":
                    want_w[pick[1]][pick[2], pick[3], pick[4]] += pr
                else:
                    want_v[pick[1]][pick[2], pick[3]] += pr
            for (s, k) in leaves:
                for d in g.scopes[s]:
                    want_tot[d, g.replica[s], k] += pr
                    want_num[d, g.replica[s], k] += pr * x[b, d, 0]
    stats, logp = model.em_accumulate(x)
    np.testing.assert_allclose(logp, want_logp, rtol=1e-12)
    for n in range(len(model.W)):
        np.testing.assert_allclose(stats["Nw"][n], want_w[n], rtol=1e-10, atol=1e-14)
    for s in model.v:
        np.testing.assert_allclose(stats["Nv"][s], want_v[s], rtol=1e-10, atol=1e-14)
    np.testing.assert_allclose(stats["tot"], want_tot, rtol=1e-10, atol=1e-14)
    np.testing.assert_allclose(stats["num"][:, 0, :, 0, :], want_num, rtol=1e-10, atol=1e-14)


# ----------------------------------------------------------------------------- P9 monotone EM
@pytest.mark.parametrize("case", ["cfg1", "rat_gauss_masked", "pd_gauss"])
def test_full_batch_em_never_decreases_likelihood(case):
    if case == "cfg1":
        cfg, model, flat, x, mask = make_config(1)
        kwargs = {}
    elif case == "rat_gauss_masked":
        model, _, rng = make_oracle(dict(kind="rat", D=12, depth=2, R=3), 3, 1, GAUSSIAN, seed=14, leaf_range=(0, 1))
        x = rng.normal(0.5, 0.3, size=(60, 12, 1)) + 0.5 * (rng.random((60, 1, 1)) < 0.5)
        mask = (rng.random((60, 12)) < 0.7).astype(float)          # missing data: exact EM still monotone
        kwargs = dict(min_var=1e-6)
    else:
        model, _, rng = make_oracle(dict(kind="pd", H=4, W=4, deltas=[2]), 3, 2, GAUSSIAN, seed=15, leaf_range=(0, 1))
        x = rng.normal(0.5, 0.2, size=(50, 16, 2))
        mask = None
        kwargs = dict(min_var=1e-6)
    prev = -np.inf
    for it in range(12):
        stats, logp = model.em_accumulate(x, mask)
        ll = logp.sum()
        assert ll >= prev - 1e-9 * abs(prev if np.isfinite(prev) else 1.0), (it, ll, prev)
        prev = ll
        model.em_update(stats, step=1.0, **kwargs)
    first = model.logp(x, mask).sum()
    assert first >= prev
    # parameters stay valid
    for w in model.W:
        np.testing.assert_allclose(w.sum(axis=(1, 2)), 1.0, rtol=1e-12)
    for v in model.v.values():
        np.testing.assert_allclose(v.sum(axis=1), 1.0, rtol=1e-12)


def test_m_step_guards():
    model, _, rng = make_oracle(dict(kind="rat", D=4, depth=1, R=2), 2, 1, GAUSSIAN, seed=16)
    before = model.get_flat_params().copy()
    model.em_update(model.zero_stats(), step=1.0)                 # nothing accumulated: parameters are kept
    np.testing.assert_array_equal(model.get_flat_params(), before)
    x = np.full((5, 4, 1), 0.25)                                  # zero sample variance
    stats, _ = model.em_accumulate(x)
    model.em_update(stats, step=1.0, min_var=1e-4, max_var=1e-2, w_floor=1e-3)
    var = model.phi[:, :, :, 1, :] - model.phi[:, :, :, 0, :] ** 2
    np.testing.assert_allclose(var, 1e-4, rtol=1e-9)
    for w in model.W:
        assert w.min() >= 1e-3 / (1 + 4 * 1e-3) - 1e-15
        np.testing.assert_allclose(w.sum(axis=(1, 2)), 1.0, rtol=1e-12)


def test_flat_round_trip_and_chunking():
    cfg, model, flat, x, mask = make_config(1)
    np.testing.assert_array_equal(model.get_flat_params(), flat.astype(np.float64))
    s1, lp1 = model.em_accumulate(x)
    s2, lp2 = model.em_accumulate(x, chunk=7)
    np.testing.assert_allclose(model.stats_to_flat(s1), model.stats_to_flat(s2), rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(lp1, lp2, rtol=0, atol=0)
    assert model.stats_to_flat(s1).size == model.layout.n_stats
    back = model.stats_from_flat(model.stats_to_flat(s1))
    np.testing.assert_array_equal(model.stats_to_flat(back), model.stats_to_flat(s1))
    np.testing.assert_array_equal(back["num"], s1["num"])


# ----------------------------------------------------------------------------- impossible evidence (-inf)
def _impossible_models():
    """Bernoulli circuits in which variable 3 has p = 0 under every leaf entry of every replica: states with
    x_3 = 1 have probability zero and the leaf vector that holds variable 3 is -inf in all of its entries."""
    for spec, K in ((dict(kind="rat", D=6, depth=1, R=1), 3), (RAT_TINY, 4), (dict(kind="pd", H=2, W=4, deltas=[1]), 2)):
        model, _, rng = make_oracle(spec, K, 1, BERNOULLI, seed=11)
        normalise_exactly(model)
        model.phi[3] = 0.0
        yield spec, K, model, rng


def test_impossible_evidence_gives_minus_inf_and_the_rest_stays_normalised():
    """The shift of Eq. 4 when a whole input vector is -inf: the oracle's logsumexp takes shift 0 there.  Pinned by
    what does not depend on that guard: the impossible states have log-density -inf exactly, the possible ones are
    finite, and the density still sums to one over all 2^D states (so the possible states carry all the mass)."""
    for spec, K, model, rng in _impossible_models():
        D = model.g.num_vars
        X = all_binary(D)
        lp = model.logp(X)
        bad = X[:, 3, 0] == 1
        assert np.all(np.isneginf(lp[bad])) and np.all(np.isfinite(lp[~bad])), spec
        assert abs(np.exp(lp).sum() - 1.0) < 1e-12, spec
        # marginalising the impossible variable makes every state possible again, with P(x_rest) = P(x_rest, x_3 = 0)
        m = np.ones(D); m[3] = 0
        lp_m = model.logp(X, m)
        assert np.all(np.isfinite(lp_m))
        x0 = X.copy(); x0[:, 3, 0] = 0
        np.testing.assert_allclose(lp_m, model.logp(x0), rtol=0, atol=1e-12)


def test_impossible_evidence_against_an_explicit_mixture():
    """Depth-1 tree, one replica: the circuit is a mixture of K^2 products of Bernoullis; its log-density,
    written with scipy's logsumexp and the Bernoulli mass function evaluated as p^x (1-p)^(1-x), is -inf
    for the impossible rows and agrees with the oracle on the others, in one mixed batch."""
    spec, K, model, rng = next(_impossible_models())
    D = model.g.num_vars
    x = (rng.random((12, D, 1)) < 0.5).astype(float)
    x[::3, 3, 0] = 1.0                                     # every third row is impossible
    x[1::3, 3, 0] = 0.0
    (_, left, right), = model.g.partitions
    W = model.W[0][0]                                      # [K, K]
    want = np.empty(12)
    for b in range(12):
        comp = np.empty((K, K))
        for i in range(K):
            for j in range(K):
                pr = W[i, j]
                for reg, k in ((left, i), (right, j)):
                    for d in model.g.scopes[reg]:
                        p = model.phi[d, 0, model.g.replica[reg], 0, k]
                        pr *= p ** x[b, d, 0] * (1.0 - p) ** (1.0 - x[b, d, 0])     # 0 ** 0 = 1
                comp[i, j] = pr
        with np.errstate(divide="ignore"):
            want[b] = scipy.special.logsumexp(np.log(comp.ravel()))
    got = model.logp(x)
    bad = x[:, 3, 0] == 1
    assert bad.any() and (~bad).any()
    assert np.all(np.isneginf(got[bad])) and np.all(np.isneginf(want[bad]))
    np.testing.assert_allclose(got[~bad], want[~bad], rtol=1e-12)
