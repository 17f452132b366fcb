"""GPU parity of the binomial and categorical leaves (Sec. 3.4) against the oracle: log-density, EM statistics,
M-step with its projection, an epoch of stochastic EM and top-down sampling."""
import numpy as np
import pytest
import torch

import workloads
from oracle.einet import BINOMIAL, CATEGORICAL
from oracle.sampling import sample
from oracle.train import em_epoch
from tests.common import make_oracle
from tests.gpu_common import gpu_model, dev, assert_logp_close, assert_stats_close

pytestmark = pytest.mark.gpu

CASES = [
    # family, leaf_param, spec, K, C, B, mask kind
    (BINOMIAL, 1, dict(kind="rat", D=12, depth=2, R=2), 4, 1, 20, None),                 # one trial = Bernoulli
    (BINOMIAL, 7, dict(kind="rat", D=16, depth=3, R=2), 5, 2, 33, "per_sample"),         # short scopes
    (BINOMIAL, 255, dict(kind="pd", H=8, W=8, deltas=[4]), 10, 3, 40, "shared"),         # 8-bit pixels, image cells
    (BINOMIAL, 31, dict(kind="rat", D=96, depth=1, R=2), 6, 1, 130, None),               # scopes of 48, batch above 128
    (CATEGORICAL, 2, dict(kind="rat", D=12, depth=2, R=2), 4, 1, 20, None),
    (CATEGORICAL, 5, dict(kind="rat", D=16, depth=3, R=2), 7, 2, 33, "per_sample"),
    (CATEGORICAL, 256, dict(kind="pd", H=8, W=8, deltas=[4]), 8, 3, 40, "shared"),       # 8-bit pixels, image cells
    (CATEGORICAL, 16, dict(kind="rat", D=96, depth=1, R=2), 64, 1, 130, None),           # largest K
    # thousands of short leaves: the leaf kernel takes four samples per thread
    (BINOMIAL, 9, dict(kind="rat", D=512, depth=7, R=20), 8, 1, 100, "per_sample"),
    (CATEGORICAL, 4, dict(kind="rat", D=512, depth=7, R=20), 8, 1, 100, "shared"),
]


def _data(rng, family, param, B, D, C):
    if family == BINOMIAL:
        spec = dict(kind="binomial_mixture", components=3, trials=param, lo=0.1, hi=0.9)
    else:
        spec = dict(kind="categorical_mixture", components=3, values=param)
    return workloads.draw_data(rng, spec, B, D, C)


@pytest.mark.parametrize("family,param,spec,K,C,B,mask_kind", CASES)
def test_discrete_leaves_match_oracle(family, param, spec, K, C, B, mask_kind):
    seed = 900 + param + K
    print("leaf family case", family, param, spec, K, C, B, mask_kind, flush=True)
    oracle, flat, rng = make_oracle(spec, K, C, family, seed, (0.15, 0.85), leaf_param=param)
    D = oracle.g.num_vars
    x = _data(rng, family, param, B, D, C)
    mask = workloads.draw_mask(rng, None if mask_kind is None else dict(kind=mask_kind, observed_fraction=0.6), B, D)
    m = gpu_model(spec, K, C, family, B, seed, flat, param)
    ref_stats, ref_logp = oracle.em_accumulate(x, mask)
    assert_logp_close(m.logp(dev(x), dev(mask)), ref_logp)
    lp = torch.empty(B, device="cuda")
    m.em_accumulate(dev(x), dev(mask), lp)
    assert_logp_close(lp, ref_logp)
    assert_stats_close(m.stats, oracle.stats_to_flat(ref_stats), oracle.layout, m.n_params)
    kw = dict(step=0.6, w_floor=1e-9)
    m.em_update(**kw)
    oracle.em_update(ref_stats, **kw)
    ref = oracle.get_flat_params()
    got = m.params.cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(got))
    # a leaf entry whose posterior mass over the batch lies below the float32 range (with 255 trials the
    # log-densities of the entries differ by hundreds) has statistics 0 on the GPU and keeps its parameters,
    # while the float64 oracle still forms the ratio of two tiny numbers: such entries are not comparable
    lay = oracle.layout
    alive = np.ones(ref.size, bool)
    alive[lay.phi_off:] = np.broadcast_to(ref_stats["tot"][:, None, :, None, :] >= 1e-30, oracle.phi.shape).ravel()
    assert alive[lay.phi_off:].mean() >= 0.2
    assert np.all(np.abs(got - ref)[alive] <= (1e-3 * np.abs(ref) + 1e-7)[alive])
    oracle.set_flat_params(np.where(alive, ref, got))         # same parameters on both sides for what follows
    # the refreshed constants are in use
    assert_logp_close(m.logp(dev(x), dev(mask)), oracle.logp(x, mask))
    m.close()


@pytest.mark.parametrize("family,param", [(BINOMIAL, 20), (CATEGORICAL, 12)])
def test_epoch_with_discrete_leaves_matches_oracle(family, param):
    spec = dict(kind="pd", H=4, W=6, deltas=[2])
    oracle, flat, rng = make_oracle(spec, 5, 1, family, 41, (0.2, 0.8), leaf_param=param)
    x = _data(rng, family, param, 90, 24, 1)
    m = gpu_model(spec, 5, 1, family, 32, 41, flat, param)
    lp = torch.empty(90, device="cuda")
    m.em_epoch(dev(x), None, batch=32, step=0.5, w_floor=1e-9, logp=lp)
    ref_lp = em_epoch(oracle, x, None, batch=32, step=0.5, w_floor=1e-9)
    assert_logp_close(lp, ref_lp)
    ref = oracle.get_flat_params()
    got = m.params.cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got - ref) <= 2e-3 * np.abs(ref) + 1e-6)
    m.close()


@pytest.mark.parametrize("family,param,values", [(BINOMIAL, 15, "draw"), (BINOMIAL, 15, "mean"),
                                                 (CATEGORICAL, 9, "draw"), (CATEGORICAL, 9, "mean")])
def test_sampling_with_discrete_leaves_matches_oracle(family, param, values):
    spec = dict(kind="rat", D=18, depth=3, R=2)
    K, B = 6, 80
    oracle, flat, rng = make_oracle(spec, K, 1, family, 43, (0.2, 0.8), leaf_param=param)
    g = oracle.g
    x = _data(rng, family, param, B, 18, 1)
    mask = workloads.draw_mask(rng, dict(kind="per_sample", observed_fraction=0.4), B, 18)
    u = rng.random((g.num_partitions + g.num_regions, B), dtype=np.float32)
    noise = rng.random((B, 18, 1), dtype=np.float32) if values == "draw" else None
    m = gpu_model(spec, K, 1, family, B, 43, flat, param)
    got = m.sample(B, dev(u), dev(noise), dev(x), dev(mask)).cpu().numpy().astype(np.float64)
    ref, margin, _ = sample(oracle, B, u.astype(np.float64), None if noise is None else noise.astype(np.float64), x, mask)
    obs = np.asarray(mask, bool)
    assert np.array_equal(got[obs], x.astype(np.float64)[obs])
    if values == "draw":
        assert np.all(got == np.round(got)) and got.min() >= 0 and got.max() <= (param if family == BINOMIAL else param - 1)
    # the leaf draws are integers decided in float32 as well: agreement is asked of most samples, and of every
    # sample in mean mode whose choices at the sums were clear-cut
    same = np.all(np.abs(got - ref) <= 1e-5 * np.abs(ref) + 1e-5, axis=(1, 2))
    if values == "mean":
        assert np.all(same[margin >= 1e-5])
    assert same.mean() >= 0.9, same.mean()
    m.close()
