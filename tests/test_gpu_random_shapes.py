"""Parity on seeded random small models: structure kind, depth, sizes, K, channels, leaf family, batch and mask
are all drawn from the case number, so that shapes nobody thought of writing down are covered too. Each case
checks logP, every E-step statistic, the M-step and top-down sampling against the oracle (Sec. 3.2-3.5)."""
import numpy as np
import pytest
import torch

import workloads
from oracle.einet import BERNOULLI, BINOMIAL, CATEGORICAL, GAUSSIAN
from oracle.sampling import sample
from tests.common import make_oracle
from tests.gpu_common import assert_logp_close, assert_stats_close, dev, gpu_model

pytestmark = pytest.mark.gpu
MARGIN = 1e-5


def draw_case(case):
    r = np.random.default_rng(1000 + case)
    family = int(r.integers(0, 4))
    K = int(r.choice([1, 2, 3, 4, 5, 7, 8, 11, 12, 16, 20, 33]))
    C = int(r.choice([1, 1, 2, 3]))
    B = int(r.choice([1, 3, 16, 17, 50, 129, 200]))
    if r.random() < 0.5:
        depth = int(r.integers(1, 5))
        spec = dict(kind="rat", D=int(r.integers(2 ** depth, 2 ** depth * 6)), depth=depth, R=int(r.integers(1, 5)))
    else:
        H, W = int(r.integers(2, 13)), int(r.integers(2, 13))
        d = int(r.integers(1, max(2, min(H, W))))
        deltas = [d] if r.random() < 0.7 else [max(1, min(2 * d, max(H, W) - 1)), d]
        spec = dict(kind="pd", H=H, W=W, deltas=sorted(set(deltas), reverse=True), axes=int(r.choice([1, 2, 3, 3])))
    param = {BINOMIAL: int(r.choice([1, 5, 30])), CATEGORICAL: int(r.choice([2, 3, 9]))}.get(family, 0)
    mask_kind = str(r.choice(["none", "shared", "per_sample"]))
    return family, param, K, C, B, spec, mask_kind, int(r.integers(1, 10 ** 6))


def draw_x(rng, family, param, B, D, C):
    recipe = {BERNOULLI: dict(kind="bernoulli_iid", p=0.4),
              GAUSSIAN: dict(kind="gaussian_mixture", components=3, std=0.3),
              BINOMIAL: dict(kind="binomial_mixture", components=3, trials=param, lo=0.1, hi=0.9),
              CATEGORICAL: dict(kind="categorical_mixture", components=3, values=param)}[family]
    return workloads.draw_data(rng, recipe, B, D, C)


@pytest.mark.parametrize("case", range(40))
def test_random_model(case):
    family, param, K, C, B, spec, mask_kind, seed = draw_case(case)
    try:
        oracle, flat, rng = make_oracle(spec, K, C, family, seed, (0.15, 0.85), leaf_param=param)
    except ValueError as e:
        pytest.skip(f"not a valid structure: {e}")
    if oracle.g.num_partitions > 3000:
        pytest.skip("larger than this test is meant for")
    D = oracle.g.num_vars
    x = draw_x(rng, family, param, B, D, C)
    mask = workloads.draw_mask(rng, None if mask_kind == "none" else dict(kind=mask_kind, observed_fraction=0.6),
                               B, D)
    m = gpu_model(spec, K, C, family, B, seed, flat, param)
    try:
        ref_stats, ref_logp = oracle.em_accumulate(x, mask)
        assert_logp_close(m.logp(dev(x), dev(mask)), ref_logp)
        lp = torch.empty(B, device="cuda")
        m.em_accumulate(dev(x), dev(mask), lp)
        assert_logp_close(lp, ref_logp)
        assert_stats_close(m.stats, oracle.stats_to_flat(ref_stats), oracle.layout, m.n_params)

        kw = dict(step=0.5, min_var=1e-4, max_var=2.0, w_floor=1e-9)
        m.em_update(**kw)
        oracle.em_update(ref_stats, **kw)
        ref = oracle.get_flat_params()
        got = m.params.cpu().numpy().astype(np.float64)
        # Leaf entries whose posterior mass is below what float32 holds keep their parameters on the GPU.
        alive = np.ones(ref.size, bool)
        alive[oracle.layout.phi_off:] = np.broadcast_to(ref_stats["tot"][:, None, :, None, :] >= 1e-30,
                                                        oracle.phi.shape).ravel()
        assert np.all(np.isfinite(got))
        assert np.all(np.abs(got - ref)[alive] <= (1e-3 * np.abs(ref) + 1e-7)[alive])

        oracle.set_flat_params(flat)
        m.set_params(flat)
        u = rng.random((oracle.g.num_partitions + oracle.g.num_regions, B), dtype=np.float32)
        if mask is None:
            got_s = m.sample(B, dev(u), None)
            ref_s, margin, _ = sample(oracle, B, u.astype(np.float64), None)
        else:
            got_s = m.sample(B, dev(u), None, dev(x), dev(mask))
            ref_s, margin, _ = sample(oracle, B, u.astype(np.float64), None, x, mask)
        got_s = got_s.cpu().numpy().astype(np.float64)
        same = np.all(np.abs(got_s - ref_s) <= 1e-5 * np.abs(ref_s) + 1e-5, axis=(1, 2))
        assert np.all(same[margin >= MARGIN])
    finally:
        m.close()
