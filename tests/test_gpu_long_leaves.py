"""GPU parity of the leaf layer (Sec. 3.4) for leaves whose scopes span several staging chunks (image strips,
halves of a long variable list): log-densities through logP and the EM statistics, for every family, with and
without marginalised variables, K from 5 to 64, ragged last chunks and ragged sample groups."""
import pytest
import torch

import workloads
from oracle.einet import BERNOULLI, BINOMIAL, CATEGORICAL, GAUSSIAN
from tests.common import make_oracle
from tests.gpu_common import gpu_model, dev, assert_logp_close, assert_stats_close

pytestmark = pytest.mark.gpu

CASES = [
    # family, leaf_param, spec, K, C, B, mask kind
    (GAUSSIAN, 0, dict(kind="pd", H=32, W=32, deltas=[8], axes=2), 40, 3, 70, None),          # strips of 256 pixels: two full chunks
    (GAUSSIAN, 0, dict(kind="pd", H=48, W=44, deltas=[24]), 33, 3, 130, "per_sample"),        # five chunks, the last ragged
    (GAUSSIAN, 0, dict(kind="rat", D=2000, depth=1, R=1), 64, 1, 9, "shared"),                # widest K: four rounds per chunk
    (GAUSSIAN, 0, dict(kind="rat", D=1800, depth=1, R=2), 5, 1, 17, None),                    # narrow K: one round per chunk
    (BERNOULLI, 0, dict(kind="rat", D=2500, depth=1, R=2), 5, 1, 70, "per_sample"),
    (BERNOULLI, 0, dict(kind="rat", D=1100, depth=1, R=1), 40, 1, 8, None),
    (BINOMIAL, 31, dict(kind="rat", D=1600, depth=1, R=1), 12, 2, 33, "shared"),              # chunks of 192 variables
    (BINOMIAL, 255, dict(kind="pd", H=32, W=32, deltas=[16], axes=2), 10, 3, 20, None),       # 8-bit pixels
    (CATEGORICAL, 4, dict(kind="rat", D=1000, depth=1, R=1), 8, 1, 20, "per_sample"),         # constants indexed by the value
    (GAUSSIAN, 0, dict(kind="rat", D=771, depth=1, R=1), 40, 1, 20, "shared"),                # second chunks of one and two variables
    (GAUSSIAN, 0, dict(kind="rat", D=2000, depth=1, R=1), 1, 1, 10, None),                    # K = 1
    # few leaves, scopes of 512 to 1023 pairs, several passes of 64 samples: statistics per batch group, then summed
    (GAUSSIAN, 0, dict(kind="pd", H=32, W=32, deltas=[8], axes=2), 40, 3, 300, None),         # two groups, the second ragged
    (BERNOULLI, 0, dict(kind="rat", D=1100, depth=1, R=1), 40, 1, 500, None),                 # four groups of two passes
    (GAUSSIAN, 0, dict(kind="rat", D=1800, depth=1, R=2), 5, 1, 260, None),                   # one column tile, two groups
    (BINOMIAL, 31, dict(kind="rat", D=1200, depth=1, R=1), 12, 1, 450, None),                 # one statistic, four groups
]


def _data(rng, family, param, B, D, C):
    spec = {GAUSSIAN: dict(kind="gaussian_mixture", components=3, std=0.3),
            BERNOULLI: dict(kind="bernoulli_iid", p=0.4),
            BINOMIAL: dict(kind="binomial_mixture", components=3, trials=param, lo=0.1, hi=0.9),
            CATEGORICAL: dict(kind="categorical_mixture", components=3, values=param)}[family]
    return workloads.draw_data(rng, spec, B, D, C)


@pytest.mark.parametrize("family,param,spec,K,C,B,mask_kind", CASES)
def test_leaves_with_long_scopes_match_oracle(family, param, spec, K, C, B, mask_kind):
    print("long leaf case", family, param, spec, K, C, B, mask_kind, flush=True)
    seed = 7000 + K + B
    oracle, flat, rng = make_oracle(spec, K, C, family, seed, (0.2, 0.8), leaf_param=param)
    D = oracle.g.num_vars
    x = _data(rng, family, param, B, D, C)
    mask = workloads.draw_mask(rng, None if mask_kind is None else dict(kind=mask_kind, observed_fraction=0.6), B, D)
    m = gpu_model(spec, K, C, family, B, seed, flat, param)
    ref_stats, ref_logp = oracle.em_accumulate(x, mask)
    assert_logp_close(m.logp(dev(x), dev(mask)), ref_logp)
    lp = torch.empty(B, device="cuda")
    m.em_accumulate(dev(x), dev(mask), lp)
    assert_logp_close(lp, ref_logp)
    ref_flat = oracle.stats_to_flat(ref_stats)
    assert_stats_close(m.stats, ref_flat, oracle.layout, m.n_params)
    m.em_accumulate(dev(x), dev(mask), lp)               # added to, not overwritten
    assert_stats_close(m.stats, 2.0 * ref_flat, oracle.layout, m.n_params)
    # fewer samples on the same handle: a last group of fewer than eight
    nb = max(1, B - 3)
    mk = None if mask is None else (mask if mask.ndim == 1 else mask[:nb])
    assert_logp_close(m.logp(dev(x[:nb]), dev(mk)), oracle.logp(x[:nb], mk))
    m.close()
