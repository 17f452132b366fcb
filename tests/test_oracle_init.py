"""Pins of oracle/init.py (no GPU, no product code)."""
import numpy as np
import pytest

from oracle import structure as S
from oracle.einet import BERNOULLI, GAUSSIAN, BINOMIAL, CATEGORICAL
from oracle.init import uniforms, init_params
from tests.common import make_oracle


def test_uniforms_are_the_top_bits_of_the_splitmix64_stream():
    """Against the generator class that the published test vectors pin (tests/test_oracle_structure.py)."""
    for seed in (0, 1234567, 2 ** 64 - 5):
        r = S.SplitMix64(seed)
        want = [((r.next() >> 41) + 0.5) / 2 ** 23 for _ in range(12)]
        np.testing.assert_array_equal(uniforms(seed, 0, 12), want)
        np.testing.assert_array_equal(uniforms(seed, 7, 5), want[7:])
    u = uniforms(3, 0, 200000)
    assert u.min() > 0.0 and u.max() < 1.0
    assert np.array_equal(u, u.astype(np.float32).astype(np.float64))       # exact in float32
    assert abs(u.mean() - 0.5) < 3e-3 and abs(u.var() - 1 / 12) < 2e-3


@pytest.mark.parametrize("family,param", [(BERNOULLI, 0), (GAUSSIAN, 0), (BINOMIAL, 12), (CATEGORICAL, 5)])
def test_initial_parameters_are_valid_and_have_the_right_moments(family, param):
    model, _, _ = make_oracle(dict(kind="rat", D=32, depth=3, R=4), 8, 2, family, 3, leaf_param=param)
    flat = init_params(model, 99, 0.2, 0.7)
    model.set_flat_params(flat)
    for w in model.W:
        np.testing.assert_allclose(w.sum(axis=(1, 2)), 1.0, rtol=1e-12)
        assert w.min() > 0
    for v in model.v.values():
        np.testing.assert_allclose(v.sum(axis=1), 1.0, rtol=1e-12)
    # Dirichlet(1,..,1) over n = 64 entries: marginal mean 1/n, variance (n-1)/(n^2 (n+1))
    allw = np.concatenate([w.reshape(-1, 64) for w in model.W[1:]])
    n = 64
    assert abs(allw.mean() - 1 / n) < 1e-12
    assert abs(allw.var() / ((n - 1) / (n * n * (n + 1))) - 1.0) < 0.1
    phi = model.phi
    if family == CATEGORICAL:
        np.testing.assert_allclose(phi.sum(axis=3), 1.0, rtol=1e-12)
    else:
        first = phi[:, :, :, 0, :] / (param if family == BINOMIAL else 1.0)
        assert first.min() >= 0.2 and first.max() <= 0.7 and abs(first.mean() - 0.45) < 0.01
        if family == GAUSSIAN:
            np.testing.assert_allclose(phi[:, :, :, 1, :] - phi[:, :, :, 0, :] ** 2, 1.0, rtol=1e-12)
    assert np.all(np.isfinite(model.logp(np.zeros((2, 32, 2)))))
    # another seed gives other numbers, the same seed the same
    assert not np.array_equal(flat, init_params(model, 100, 0.2, 0.7))
    assert np.array_equal(flat, init_params(model, 99, 0.2, 0.7))
