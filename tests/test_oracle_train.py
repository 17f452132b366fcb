"""Pins of oracle/train.py against what the mathematics fixes (no GPU, no product code)."""
import numpy as np
import pytest
from scipy.stats import norm

from oracle.einet import BERNOULLI, GAUSSIAN
from oracle.train import em_epoch, mixture_logp
from tests.common import make_oracle, all_binary, normalise_exactly

ONE_ENTRY = dict(kind="rat", D=4, depth=1, R=1)      # K = 1, one replica: a fully factorised density


def _one_entry_model(family, seed):
    model, flat, rng = make_oracle(ONE_ENTRY, 1, 1, family, seed, (0.2, 0.8))
    return model, rng


@pytest.mark.parametrize("N,batch", [(20, 5), (23, 5), (7, 16)])
def test_epoch_on_a_factorised_gaussian_is_a_moving_average_of_minibatch_moments(N, batch):
    """With one entry per sum and leaf every posterior is 1, so Eq. 7 gives the mini-batch moments and
    Eq. 8-9 an exponential moving average of them; logP is a sum of univariate normal log-densities
    under the parameters in force before the mini-batch's update."""
    model, rng = _one_entry_model(GAUSSIAN, 3)
    x = rng.normal(0.3, 1.5, size=(N, 4, 1))
    lam = 0.3
    mu = model.phi[:, 0, 0, 0, 0].copy()
    m2 = model.phi[:, 0, 0, 1, 0].copy()
    expect_lp = np.empty(N)
    for b0 in range(0, N, batch):
        xb = x[b0:b0 + batch, :, 0]
        expect_lp[b0:b0 + batch] = norm.logpdf(xb, mu, np.sqrt(m2 - mu ** 2)).sum(axis=1)
        mu = (1 - lam) * mu + lam * xb.mean(axis=0)
        m2 = (1 - lam) * m2 + lam * (xb ** 2).mean(axis=0)
    lp = em_epoch(model, x, None, batch=batch, step=lam)
    np.testing.assert_allclose(model.phi[:, 0, 0, 0, 0], mu, rtol=1e-12)
    np.testing.assert_allclose(model.phi[:, 0, 0, 1, 0], m2, rtol=1e-12)
    np.testing.assert_allclose(lp, expect_lp, rtol=1e-11)


def test_epoch_projects_the_variance_after_every_update():
    """Sec. 4.2: the variance is brought back into [min_var, max_var] after each update, so the next
    mini-batch already sees the projected value."""
    model, rng = _one_entry_model(GAUSSIAN, 4)
    x = rng.normal(0.0, 3.0, size=(12, 4, 1))
    lam, lo, hi = 0.5, 0.5, 2.0
    mu = model.phi[:, 0, 0, 0, 0].copy()
    m2 = model.phi[:, 0, 0, 1, 0].copy()
    for b0 in range(0, 12, 4):
        xb = x[b0:b0 + 4, :, 0]
        mu = (1 - lam) * mu + lam * xb.mean(axis=0)
        m2 = (1 - lam) * m2 + lam * (xb ** 2).mean(axis=0)
        m2 = mu ** 2 + np.clip(m2 - mu ** 2, lo, hi)
    em_epoch(model, x, None, batch=4, step=lam, min_var=lo, max_var=hi)
    np.testing.assert_allclose(model.phi[:, 0, 0, 0, 0], mu, rtol=1e-12)
    np.testing.assert_allclose(model.phi[:, 0, 0, 1, 0], m2, rtol=1e-12)
    var = model.phi[:, 0, 0, 1, 0] - model.phi[:, 0, 0, 0, 0] ** 2
    assert np.all(var >= lo - 1e-12) and np.all(var <= hi + 1e-12)
    assert np.any(np.isclose(var, hi))            # the projection was active


def test_epoch_with_a_per_sample_mask_uses_the_rows_of_its_minibatch():
    """Bernoulli, one entry: a missing value contributes the current parameter as its expectation, so a
    mini-batch of n samples with observed set O gives hat = (sum_O x + (n - |O|) p_old) / n."""
    model, rng = _one_entry_model(BERNOULLI, 5)
    N, batch, lam = 14, 4, 0.7
    x = (rng.random((N, 4, 1)) < 0.4).astype(np.float64)
    mask = rng.random((N, 4)) < 0.6
    p = model.phi[:, 0, 0, 0, 0].copy()
    for b0 in range(0, N, batch):
        xb, mb = x[b0:b0 + batch, :, 0], mask[b0:b0 + batch]
        n = xb.shape[0]
        hat = ((xb * mb).sum(axis=0) + (n - mb.sum(axis=0)) * p) / n
        p = (1 - lam) * p + lam * hat
    em_epoch(model, x, mask, batch=batch, step=lam)
    np.testing.assert_allclose(model.phi[:, 0, 0, 0, 0], p, rtol=1e-12)


def test_full_batch_epochs_never_decrease_the_likelihood():
    model, flat, rng = make_oracle(dict(kind="rat", D=8, depth=2, R=2), 3, 1, BERNOULLI, 6)
    x = (rng.random((60, 8, 1)) < 0.35).astype(np.float64)
    last = -np.inf
    for _ in range(6):
        ll = em_epoch(model, x, None, batch=60, step=1.0).sum()
        assert ll >= last - 1e-9
        last = ll


def test_mixture_of_normalised_circuits_is_normalised_and_reduces_to_its_component():
    X = all_binary(8)
    comps = []
    for seed in (11, 12, 13):
        model, _, _ = make_oracle(dict(kind="rat", D=8, depth=2, R=2), 2, 1, BERNOULLI, seed)
        normalise_exactly(model)
        comps.append(model.logp(X))
    comps = np.stack(comps)
    coef = np.array([0.2, 0.5, 0.3])
    mix = mixture_logp(comps, np.log(coef))
    assert abs(np.exp(mix).sum() - 1.0) < 1e-12
    np.testing.assert_allclose(np.exp(mix), (coef[:, None] * np.exp(comps)).sum(axis=0), rtol=1e-12)
    np.testing.assert_allclose(mixture_logp(comps[1:2], [0.0]), comps[1], rtol=0, atol=1e-13)
    # a component that gives zero probability does not disturb the others; nothing left gives -inf
    holes = comps.copy()
    holes[0, :5] = -np.inf
    got = mixture_logp(holes, np.log(coef))
    np.testing.assert_allclose(np.exp(got[:5]), (coef[1:, None] * np.exp(comps[1:, :5])).sum(axis=0), rtol=1e-12)
    holes[:, 0] = -np.inf
    assert mixture_logp(holes, np.log(coef))[0] == -np.inf
    # far below the float64 exponent range the shift keeps the result finite
    deep = comps - 5000.0
    np.testing.assert_allclose(mixture_logp(deep, np.log(coef)), mix - 5000.0, rtol=1e-12)
