"""Float64 oracle of the random initialisation the library offers (einet_init_params).

TEST INFRASTRUCTURE ONLY (see the package docstring).  The paper does not prescribe an
initialisation; the library's is the customary one for circuits: every normalised weight
vector is drawn from the flat Dirichlet distribution and the leaf parameters uniformly
from a range.  It is specified through a counter-based generator so that this oracle and
the kernel produce the same numbers:

    u(p) = (top 23 bits of SplitMix64 output number p + 1 of the stream started at `seed`
            + 1/2) / 2^23,          p = position of the parameter in the flat buffer

  * weight row (the K*K weights of a sum entry, or the C weights of a mixing entry):
    e_p = -log u(p), w_p = e_p / sum of the row's e  (normalised unit exponentials are
    Dirichlet(1, ..., 1))
  * Bernoulli p, Gaussian mean, binomial E[x] / N: lo + (hi - lo) * u(p), the Gaussian second
    moment is mean^2 + 1 (variance 1)
  * categorical probabilities: as a weight row over the V values of one (variable, channel,
    replica, entry).

Pinned by tests/test_oracle_init.py: the generator against the published SplitMix64
vectors, rows on the simplex, moments of the uniform and of the Dirichlet marginals.
"""
import numpy as np

from .einet import GAUSSIAN, BINOMIAL, CATEGORICAL
from .structure import MASK64

_GAMMA = 0x9E3779B97F4A7C15


def uniforms(seed, first, count):
    """u(p) for p = first .. first + count - 1, as float64 (exactly representable in float32)."""
    p = np.arange(first + 1, first + count + 1, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = np.uint64(seed & MASK64) + p * np.uint64(_GAMMA)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        z = z ^ (z >> np.uint64(31))
    return ((z >> np.uint64(41)).astype(np.float64) + 0.5) / 2.0 ** 23


def init_params(model, seed, lo, hi):
    """Flat float64 parameter vector for `model` (an OracleEiNet gives the layout and the shapes)."""
    g, K, lay = model.g, model.K, model.layout
    out = np.zeros(lay.n_params)

    def rows(off, n_rows, row_len):
        e = -np.log(uniforms(seed, off, n_rows * row_len)).reshape(n_rows, row_len)
        out[off: off + n_rows * row_len] = (e / e.sum(axis=1, keepdims=True)).ravel()

    for n, (parent, _, _) in enumerate(g.partitions):
        rows(lay.w_off[n], g.k_out(parent, K), K * K)
    for s, off in lay.v_off.items():
        rows(off, g.k_out(s, K), len(g.children[s]))
    D, C, R, T = g.num_vars, model.C, g.num_replica, model.T
    u = uniforms(seed, lay.phi_off, D * C * R * T * K).reshape(D, C, R, T, K)
    if model.family == CATEGORICAL:
        e = -np.log(u)
        phi = e / e.sum(axis=3, keepdims=True)
    else:
        phi = np.zeros((D, C, R, T, K))
        first = lo + (hi - lo) * u[:, :, :, 0, :]
        phi[:, :, :, 0, :] = first
        if model.family == GAUSSIAN:
            phi[:, :, :, 1, :] = first ** 2 + 1.0
        elif model.family == BINOMIAL:
            phi[:, :, :, 0, :] = model.leaf_param * first
    out[lay.phi_off:] = phi.ravel()
    return out
