"""Seeded random inputs: parameters, data and masks.

Every function takes a ``numpy.random.Generator`` and plain shape
descriptions; nothing here knows how a circuit is evaluated.  A workload draws
from one generator, ``default_rng(config_seed(i))``, in the fixed order
parameters -> data -> mask.  (The structure seed of the random binary trees is
``config_seed(i)`` itself.)
"""
import numpy as np

from .configs import BERNOULLI, GAUSSIAN, BINOMIAL, CATEGORICAL


def config_seed(i):
    """Seed of configuration i (1-based)."""
    return 20040623 + i


def draw_params(rng, n_params, weight_blocks, phi_off, phi_shape, family, leaf_range, leaf_param=0):
    """Flat float32 parameter vector.

    weight_blocks : iterable of (offset, rows, row_len); every row is drawn
                    from Dirichlet(1,...,1) (normalised unit exponentials)
    phi_shape     : (D, C, R, T, K), stored at phi_off; Bernoulli: p ~ U(lo,hi);
                    Gaussian: mean ~ U(lo,hi), variance 1, stored in
                    expectation form (mean, mean^2 + variance); binomial with
                    leaf_param trials: expected count leaf_param * U(lo,hi);
                    categorical with T = leaf_param values: probabilities from
                    Dirichlet(1,...,1) over the T axis
    """
    out = np.zeros(n_params, dtype=np.float32)
    for off, rows, row_len in weight_blocks:
        e = rng.standard_exponential((rows, row_len))
        e /= e.sum(axis=1, keepdims=True)
        out[off: off + rows * row_len] = e.ravel().astype(np.float32)
    D, C, R, T, K = phi_shape
    lo, hi = leaf_range
    phi = np.zeros((D, C, R, T, K))
    if family == CATEGORICAL:
        assert T == leaf_param
        e = rng.standard_exponential((D, C, R, T, K))
        phi = e / e.sum(axis=3, keepdims=True)
    else:
        first = rng.uniform(lo, hi, size=(D, C, R, K))
        phi[:, :, :, 0, :] = first
        if family == GAUSSIAN:
            assert T == 2
            phi[:, :, :, 1, :] = first ** 2 + 1.0
        elif family == BINOMIAL:
            assert T == 1
            phi[:, :, :, 0, :] = leaf_param * first
        else:
            assert family == BERNOULLI and T == 1
    out[phi_off: phi_off + phi.size] = phi.ravel().astype(np.float32)
    return out


def draw_data(rng, spec, B, D, C):
    """float32 [B, D, C] samples from the seeded generator named in spec."""
    kind = spec["kind"]
    if kind == "bernoulli_iid":
        return (rng.random((B, D, C)) < spec["p"]).astype(np.float32)
    if kind == "bernoulli_mixture":
        M = spec["components"]
        pi = rng.dirichlet(np.ones(M))
        q = rng.uniform(spec["lo"], spec["hi"], size=(M, D, C))
        z = rng.choice(M, size=B, p=pi)
        return (rng.random((B, D, C)) < q[z]).astype(np.float32)
    if kind == "gaussian_mixture":
        M = spec["components"]
        pi = rng.dirichlet(np.ones(M))
        mu = rng.uniform(0.0, 1.0, size=(M, D, C))
        z = rng.choice(M, size=B, p=pi)
        x = mu[z] + spec["std"] * rng.standard_normal((B, D, C))
        return np.clip(x, 0.0, 1.0).astype(np.float32)
    if kind == "binomial_mixture":
        M, N = spec["components"], spec["trials"]
        pi = rng.dirichlet(np.ones(M))
        q = rng.uniform(spec["lo"], spec["hi"], size=(M, D, C))
        z = rng.choice(M, size=B, p=pi)
        return rng.binomial(N, q[z]).astype(np.float32)
    if kind == "categorical_mixture":
        M, V = spec["components"], spec["values"]
        pi = rng.dirichlet(np.ones(M))
        centre = rng.integers(0, V, size=(M, D, C))
        z = rng.choice(M, size=B, p=pi)
        jitter = rng.integers(-1, 2, size=(B, D, C))
        return np.clip(centre[z] + jitter, 0, V - 1).astype(np.float32)
    if kind == "gaussian_noise":
        return rng.standard_normal((B, D, C)).astype(np.float32)
    raise ValueError(kind)


def draw_mask(rng, spec, B, D):
    """uint8 mask, 1 = observed, 0 = marginalised; [D] (shared) or [B, D]."""
    if spec is None:
        return None
    n_obs = int(round(spec["observed_fraction"] * D))
    if spec["kind"] == "shared":
        m = np.zeros(D, dtype=np.uint8)
        m[rng.permutation(D)[:n_obs]] = 1
        return m
    if spec["kind"] == "per_sample":
        m = np.zeros((B, D), dtype=np.uint8)
        for b in range(B):
            m[b, rng.permutation(D)[:n_obs]] = 1
        return m
    raise ValueError(spec["kind"])
