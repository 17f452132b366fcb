"""Pins of oracle/sampling.py against what the mathematics fixes (no GPU, no product code)."""
import numpy as np
import pytest

from oracle import structure as S
from oracle.einet import OracleEiNet, BERNOULLI, GAUSSIAN
from oracle.sampling import sample, choose
from tests.common import make_oracle, all_binary, normalise_exactly


def test_choice_is_the_inverse_cdf_with_the_documented_tie_rule():
    w = np.array([0.125, 0.0, 0.25, 0.25, 0.375])             # dyadic: the running sums .125 .125 .375 .625 1 are exact
    us = (0.0, 0.1, 0.125, 0.3, 0.375, 0.6, 0.625, 0.999)
    assert [choose(w, u)[0] for u in us] == [0, 0, 2, 2, 3, 3, 4, 4]     # a boundary belongs to the next entry
    assert choose(w * 7.0, 0.3)[0] == 2                       # unnormalised weights
    t, margin = choose(w, 0.5)
    assert t == 3 and abs(margin - 0.125) < 1e-15             # 0.5 sits 0.125 from both 0.375 and 0.625
    assert choose(np.array([0.5, 0.5, 0.0]), 1.0 - 1e-17)[0] == 1   # never an entry of weight zero


def _two_leaf_model(family, W, means):
    """One partition over two variables, K = 2, entry k of variable d has mean means[d][k]."""
    g = S.RegionGraph(2)
    root = g.add_region((0, 1))
    a = g.add_region((0,))
    b = g.add_region((1,))
    g.add_partition(root, a, b)
    g.replica[a] = g.replica[b] = 0
    g.num_replica = 1
    m = OracleEiNet(g, 2, 1, family)
    flat = np.zeros(m.layout.n_params)
    m.set_flat_params(flat)
    m.W[0] = np.asarray(W, dtype=np.float64).reshape(1, 2, 2)
    m.phi = np.zeros((2, 1, 1, m.T, 2))
    for d in range(2):
        for k in range(2):
            m.phi[d, 0, 0, 0, k] = means[d][k]
            if family == GAUSSIAN:
                m.phi[d, 0, 0, 1, k] = means[d][k] ** 2 + 0.25      # sd 0.5
    return m


def test_pairs_are_numbered_left_entry_major_and_each_child_gets_its_own_entry():
    """Hand-computed: W = [[.1,.2],[.3,.4]] has running sums .1 .3 .6 1.0 over (0,0),(0,1),(1,0),(1,1); in mean
    mode the sample shows which entry each child used."""
    m = _two_leaf_model(GAUSSIAN, [[0.1, 0.2], [0.3, 0.4]], [[10.0, 20.0], [-1.0, -2.0]])
    u = np.zeros((1 + 3, 4))
    u[0] = [0.05, 0.25, 0.5, 0.7]
    out, margin, paths = sample(m, 4, u, noise=None)
    np.testing.assert_array_equal(out[:, :, 0], [[10.0, -1.0], [10.0, -2.0], [20.0, -1.0], [20.0, -2.0]])
    assert paths == [[(0, 0, 0)], [(0, 0, 1)], [(0, 1, 0)], [(0, 1, 1)]]
    np.testing.assert_allclose(margin, [0.05, 0.05, 0.1, 0.1], atol=1e-12)


def test_evidence_reweights_the_pairs_by_the_children_densities():
    """Observing variable 0 at the mean of its entry 1 (sd 0.5, the other mean 20 sd away) makes pairs with i = 0
    impossible: the choice is between (1,0) and (1,1) with odds 3 : 4, whatever u."""
    m = _two_leaf_model(GAUSSIAN, [[0.1, 0.2], [0.3, 0.4]], [[10.0, 20.0], [-1.0, -2.0]])
    x = np.zeros((2, 2, 1))
    x[:, 0, 0] = 20.0
    u = np.zeros((4, 2))
    u[0] = [0.42, 0.44]                                        # boundary at 3/7 = 0.4286
    out, _, paths = sample(m, 2, u, noise=None, x=x, mask=np.array([1, 0]))
    assert paths == [[(0, 1, 0)], [(0, 1, 1)]]
    np.testing.assert_array_equal(out[:, :, 0], [[20.0, -1.0], [20.0, -2.0]])      # evidence kept


@pytest.mark.parametrize("family", [BERNOULLI, GAUSSIAN])
def test_one_entry_circuit_samples_every_variable_independently(family):
    model, flat, rng = make_oracle(dict(kind="rat", D=6, depth=2, R=1), 1, 2, family, 8, (0.2, 0.8))
    B = 50
    u = rng.random((model.g.num_partitions + model.g.num_regions, B))
    noise = rng.standard_normal((B, 6, 2)) if family == GAUSSIAN else rng.random((B, 6, 2))
    out, _, _ = sample(model, B, u, noise)
    p = model.phi[:, :, 0, 0, 0]
    if family == GAUSSIAN:
        sd = np.sqrt(model.phi[:, :, 0, 1, 0] - p ** 2)
        np.testing.assert_allclose(out, p[None] + sd[None] * noise, rtol=1e-13)
    else:
        np.testing.assert_array_equal(out, (noise < p[None]).astype(np.float64))
    means, _, _ = sample(model, B, u, None)
    np.testing.assert_array_equal(means, np.broadcast_to(p[None], (B, 6, 2)))
    # evidence is kept, the rest is drawn
    x = rng.random((B, 6, 2))
    mask = np.array([1, 0, 0, 1, 1, 0])
    cond, _, _ = sample(model, B, u, noise, x=x, mask=mask)
    np.testing.assert_array_equal(cond[:, mask == 1], x[:, mask == 1])
    np.testing.assert_array_equal(cond[:, mask == 0], out[:, mask == 0])


def _chi_square(counts, probs):
    n = counts.sum()
    return float(((counts - n * probs) ** 2 / (n * probs)).sum())


def test_ancestral_samples_follow_the_distribution_of_the_circuit():
    """Frequencies of the 2^6 states over 30000 samples against exp(logP) of every state (chi-square with 63
    degrees of freedom: mean 63, standard deviation 11.2)."""
    model, flat, rng = make_oracle(dict(kind="rat", D=6, depth=2, R=2), 2, 1, BERNOULLI, 21, (0.15, 0.85))
    normalise_exactly(model)
    probs = np.exp(model.logp(all_binary(6)))
    assert abs(probs.sum() - 1.0) < 1e-12
    B = 30000
    u = rng.random((model.g.num_partitions + model.g.num_regions, B))
    out, _, _ = sample(model, B, u, rng.random((B, 6, 1)))
    states = (out[:, :, 0].astype(np.int64) << np.arange(6)[None, :]).sum(axis=1)
    counts = np.bincount(states, minlength=64).astype(np.float64)
    assert _chi_square(counts, probs) < 63 + 5 * 11.2
    # and a wrong distribution would be noticed: against the uniform one the statistic explodes
    assert _chi_square(counts, np.full(64, 1 / 64)) > 1000


def test_conditional_samples_follow_eq1():
    """Three of six variables observed: the frequencies of the other three (8 states, 7 degrees of freedom: mean 7,
    standard deviation 3.7) against the conditional of Eq. 1 computed from two marginals."""
    model, flat, rng = make_oracle(dict(kind="pd", H=2, W=3, deltas=[1]), 3, 1, BERNOULLI, 22, (0.1, 0.9))
    normalise_exactly(model)
    mask = np.array([1, 0, 1, 0, 0, 1])
    ev = np.array([1.0, 0.0, 0.0, 0.0, 0.0, 1.0])
    B = 20000
    x = np.broadcast_to(ev[None, :, None], (B, 6, 1)).copy()
    u = rng.random((model.g.num_partitions + model.g.num_regions, B))
    out, _, _ = sample(model, B, u, rng.random((B, 6, 1)), x=x, mask=mask)
    np.testing.assert_array_equal(out[:, mask == 1, 0], np.broadcast_to(ev[mask == 1], (B, 3)))
    q = np.nonzero(mask == 0)[0]
    states = (out[:, q, 0].astype(np.int64) << np.arange(3)[None, :]).sum(axis=1)
    counts = np.bincount(states, minlength=8).astype(np.float64)
    full = np.broadcast_to(ev[None, :, None], (8, 6, 1)).copy()
    full[:, q, 0] = (np.arange(8)[:, None] >> np.arange(3)[None, :]) & 1
    cond = np.exp(model.logp(full) - model.logp(full[:1], mask)[0])
    assert abs(cond.sum() - 1.0) < 1e-12
    assert _chi_square(counts, cond) < 7 + 5 * 3.7


def test_choose_other_side_and_flipped_descent():
    """The near-tie helper used by the GPU comparison: the neighbour across the nearer boundary, by hand."""
    from oracle.sampling import choose
    w = [1.0, 1.0, 0.0, 2.0]                               # running sums 1, 2, 2, 4
    assert choose(w, 0.2500001)[0] == 1 and choose(w, 0.2500001, other_side=True)[0] == 0
    assert choose(w, 0.4999999)[0] == 1 and choose(w, 0.4999999, other_side=True)[0] == 3    # skips the zero weight
    assert choose(w, 0.1)[0] == 0 and choose(w, 0.1, other_side=True)[0] == 0                # nothing below index 0
    assert choose(w, 0.9)[0] == 3 and choose(w, 0.9, other_side=True)[0] == 3                # nothing above the last
    # a flipped descent is the unflipped one up to the flipped choice, and a valid sample afterwards
    model, _, rng = make_oracle(dict(kind="rat", D=8, depth=2, R=2), 3, 1, BERNOULLI, 11)
    g = model.g
    u = rng.random((g.num_partitions + g.num_regions, 4))
    noise = rng.random((4, 8, 1))
    ref, margin, paths = sample(model, 4, u, noise)
    # with tie_margin = 1 every choice counts as a near-tie: flip number j changes choice j and keeps those before it
    alt, _, apaths = sample(model, 4, u, noise, only=[2], flip={2: 1}, tie_margin=1.0)
    assert apaths[0] == [] and apaths[2] != paths[2]
    assert np.all((alt[2] == 0.0) | (alt[2] == 1.0))
    same_again, _, p2 = sample(model, 4, u, noise, only=[2], flip={2: 99}, tie_margin=1.0)     # no such choice: unchanged
    assert p2[2] == paths[2] and np.array_equal(same_again[2], ref[2])
