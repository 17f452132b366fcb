"""Seeded random inputs: parameters, data and masks.

Every function takes a ``numpy.random.Generator`` and plain shape
descriptions; nothing here knows how a circuit is evaluated.  A workload draws
from one generator, ``default_rng(config_seed(i))``, in the fixed order
parameters -> data -> mask.  (The structure seed of the random binary trees is
``config_seed(i)`` itself.)
"""
import numpy as np

from .configs import BERNOULLI, GAUSSIAN


def config_seed(i):
    """Seed of configuration i (1-based)."""
    return 20040623 + i


def draw_params(rng, n_params, weight_blocks, phi_off, phi_shape, family, leaf_range):
    """Flat float32 parameter vector.

    weight_blocks : iterable of (offset, rows, row_len); every row is drawn
                    from Dirichlet(1,...,1) (normalised unit exponentials)
    phi_shape     : (D, C, R, T, K), stored at phi_off; Bernoulli: p ~ U(lo,hi);
                    Gaussian: mean ~ U(lo,hi), variance 1, stored in
                    expectation form (mean, mean^2 + variance)
    """
    out = np.zeros(n_params, dtype=np.float32)
    for off, rows, row_len in weight_blocks:
        e = rng.standard_exponential((rows, row_len))
        e /= e.sum(axis=1, keepdims=True)
        out[off: off + rows * row_len] = e.ravel().astype(np.float32)
    D, C, R, T, K = phi_shape
    lo, hi = leaf_range
    first = rng.uniform(lo, hi, size=(D, C, R, K))
    phi = np.zeros((D, C, R, T, K))
    phi[:, :, :, 0, :] = first
    if family == GAUSSIAN:
        assert T == 2
        phi[:, :, :, 1, :] = first ** 2 + 1.0
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
