"""Pins of the binomial and categorical leaves of the oracle (Sec. 3.4: exponential families in expectation
parameters) against library routines, brute force and closed forms (no GPU, no product code)."""
import itertools

import numpy as np
import pytest
import scipy.stats

from oracle.einet import BINOMIAL, CATEGORICAL, ef_log_density
from oracle.sampling import sample
from oracle.train import em_epoch
from tests.common import make_oracle, normalise_exactly


def test_binomial_log_density_is_scipys():
    rng = np.random.default_rng(0)
    N = 17
    p = rng.uniform(0.05, 0.95, size=(5, 3))
    x = rng.integers(0, N + 1, size=(5, 3)).astype(np.float64)
    got = ef_log_density(BINOMIAL, x, np.stack([N * p]), N)
    np.testing.assert_allclose(got, scipy.stats.binom.logpmf(x, N, p), rtol=1e-12)


def test_categorical_log_density_is_the_log_of_the_selected_probability():
    rng = np.random.default_rng(1)
    V = 6
    phi = rng.dirichlet(np.ones(V), size=(4, 5)).transpose(2, 0, 1)      # [V, 4, 5]
    x = rng.integers(0, V, size=(4, 5))
    got = ef_log_density(CATEGORICAL, x.astype(np.float64), phi, V)
    want = np.log(np.take_along_axis(phi, x[None], axis=0)[0])
    np.testing.assert_allclose(got, want, rtol=1e-13)
    zero = phi.copy()
    zero[2] = 0.0
    assert np.all(np.isneginf(ef_log_density(CATEGORICAL, np.full((4, 5), 2.0), zero, V)))


@pytest.mark.parametrize("family,param,n_values", [(BINOMIAL, 3, 4), (CATEGORICAL, 3, 3)])
def test_circuit_with_discrete_leaves_is_normalised(family, param, n_values):
    model, flat, rng = make_oracle(dict(kind="rat", D=4, depth=2, R=2), 3, 1, family, 31, (0.2, 0.8), leaf_param=param)
    normalise_exactly(model)
    if family == CATEGORICAL:
        model.phi /= model.phi.sum(axis=3, keepdims=True)
    states = np.array(list(itertools.product(range(n_values), repeat=4)), dtype=np.float64)[:, :, None]
    assert abs(np.exp(model.logp(states)).sum() - 1.0) < 1e-12
    # marginalising a variable = summing it out
    mask = np.array([1, 0, 1, 1])
    sub = states[states[:, 1, 0] == 0]
    summed = np.zeros(len(sub))
    for v in range(n_values):
        full = sub.copy()
        full[:, 1, 0] = v
        summed += np.exp(model.logp(full))
    np.testing.assert_allclose(np.exp(model.logp(sub, mask)), summed, rtol=1e-12)


@pytest.mark.parametrize("family,param", [(BINOMIAL, 9), (CATEGORICAL, 5)])
def test_one_entry_circuit_learns_moments_or_frequencies_in_one_step(family, param):
    model, flat, rng = make_oracle(dict(kind="rat", D=5, depth=2, R=1), 1, 2, family, 32, (0.3, 0.7), leaf_param=param)
    n_val = param + 1 if family == BINOMIAL else param
    x = rng.integers(0, n_val, size=(400, 5, 2)).astype(np.float64)
    stats, _ = model.em_accumulate(x)
    model.em_update(stats, step=1.0)
    if family == BINOMIAL:
        np.testing.assert_allclose(model.phi[:, :, 0, 0, 0], x.mean(axis=0), rtol=1e-12)
    else:
        for v in range(param):
            np.testing.assert_allclose(model.phi[:, :, 0, v, 0], (x == v).mean(axis=0), rtol=1e-12)
    # with missing values the current parameter stands in (exact EM for missing data): fixed point at the
    # observed moments
    mask = rng.random((400, 5)) < 0.5
    before = model.phi.copy()
    stats, _ = model.em_accumulate(x, mask)
    model.em_update(stats, step=1.0)
    for d in range(5):
        obs = x[mask[:, d], d]                                  # [n_obs, 2]
        n_obs, n = obs.shape[0], 400
        if family == BINOMIAL:
            want = (obs.sum(axis=0) + (n - n_obs) * before[d, :, 0, 0, 0]) / n
            np.testing.assert_allclose(model.phi[d, :, 0, 0, 0], want, rtol=1e-12)
        else:
            for v in range(param):
                want = ((obs == v).sum(axis=0) + (n - n_obs) * before[d, :, 0, v, 0]) / n
                np.testing.assert_allclose(model.phi[d, :, 0, v, 0], want, rtol=1e-12)


@pytest.mark.parametrize("family,param", [(BINOMIAL, 6), (CATEGORICAL, 4)])
def test_full_batch_em_is_monotone_with_discrete_leaves(family, param):
    model, flat, rng = make_oracle(dict(kind="pd", H=2, W=4, deltas=[1]), 3, 1, family, 33, (0.2, 0.8), leaf_param=param)
    n_val = param + 1 if family == BINOMIAL else param
    x = rng.integers(0, n_val, size=(80, 8, 1)).astype(np.float64)
    last = -np.inf
    for _ in range(8):
        ll = em_epoch(model, x, None, batch=80, step=1.0).sum()
        assert ll >= last - 1e-9
        last = ll


def test_projection_keeps_probabilities_off_the_boundary():
    model, flat, rng = make_oracle(dict(kind="rat", D=4, depth=1, R=1), 2, 1, CATEGORICAL, 34, leaf_param=4)
    x = np.zeros((30, 4, 1))                                   # only value 0 ever occurs
    stats, _ = model.em_accumulate(x)
    model.em_update(stats, step=1.0)
    np.testing.assert_allclose(model.phi.sum(axis=3), 1.0, rtol=1e-12)
    np.testing.assert_allclose(model.phi[:, :, :, 1:, :], 1e-6 / (1.0 + 3e-6), rtol=1e-9)
    assert np.all(np.isfinite(model.logp(np.full((2, 4, 1), 3.0))))
    bino, _, _ = make_oracle(dict(kind="rat", D=4, depth=1, R=1), 2, 1, BINOMIAL, 35, leaf_param=5)
    stats, _ = bino.em_accumulate(np.full((30, 4, 1), 5.0))
    bino.em_update(stats, step=1.0)
    np.testing.assert_allclose(bino.phi, 5.0 * (1.0 - 1e-6), rtol=1e-12)


@pytest.mark.parametrize("family,param", [(BINOMIAL, 12), (CATEGORICAL, 7)])
def test_discrete_leaves_are_sampled_by_inverse_cdf(family, param):
    model, flat, rng = make_oracle(dict(kind="rat", D=4, depth=1, R=1), 1, 1, family, 36, (0.2, 0.8), leaf_param=param)
    B = 300
    u = rng.random((model.g.num_partitions + model.g.num_regions, B))
    noise = rng.random((B, 4, 1))
    out, _, _ = sample(model, B, u, noise)
    for d in range(4):
        if family == BINOMIAL:
            want = scipy.stats.binom.ppf(noise[:, d, 0], param, model.phi[d, 0, 0, 0, 0] / param)
        else:
            want = np.searchsorted(np.cumsum(model.phi[d, 0, 0, :, 0]), noise[:, d, 0], side="right")
        np.testing.assert_array_equal(out[:, d, 0], want)
    means, _, _ = sample(model, B, u, None)
    if family == BINOMIAL:
        np.testing.assert_allclose(means[0, :, 0], model.phi[:, 0, 0, 0, 0], rtol=1e-13)
    else:
        np.testing.assert_allclose(means[0, :, 0], (np.arange(param)[None] * model.phi[:, 0, 0, :, 0]).sum(axis=1), rtol=1e-13)
