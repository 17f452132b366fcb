"""GPU parity of the einsum kernels with specialised waves over every K they are instantiated for (multiples of 8:
bottom-up to 48, top-down to 40; K = 48 takes the new kernel one way and the 16x16x4 kernel the other), with batches
that span several chunks of 128 samples and a ragged last one, with statistics added to (two E-steps in a row),
overwritten (E-step after an M-step) and mixing weights in play (regions with several partitions); and of the
top-down kernels that add up the posterior blocks of a region's only parent themselves (random binary trees), with
the number of posterior-assembly launches each case should still need."""
import numpy as np
import pytest
import torch

import workloads
from oracle.einet import BERNOULLI, GAUSSIAN
from tests.common import make_oracle
from tests.gpu_common import gpu_model, dev, assert_logp_close, assert_stats_close

pytestmark = pytest.mark.gpu

CASES = [
    # spec, K, C, family, B
    (dict(kind="rat", D=32, depth=3, R=2), 8, 1, BERNOULLI, 300),          # three chunks, the last ragged
    (dict(kind="pd", H=8, W=4, deltas=[4, 2]), 16, 1, BERNOULLI, 129),     # one sample beyond a chunk
    (dict(kind="pd", H=8, W=8, deltas=[4]), 24, 1, GAUSSIAN, 200),         # two 16-column statistics tiles, one half used
    (dict(kind="pd", H=6, W=6, deltas=[2]), 32, 1, GAUSSIAN, 77),          # one 32-column tile, nothing left over
    (dict(kind="rat", D=16, depth=2, R=2), 40, 2, GAUSSIAN, 1),            # a single sample
    (dict(kind="pd", H=6, W=4, deltas=[2]), 40, 1, BERNOULLI, 260),        # K = 40 with chunks
    (dict(kind="rat", D=24, depth=2, R=3), 48, 1, GAUSSIAN, 130),          # new kernel bottom-up, 16x16x4 kernel top-down
    # few items and many chunks: the chunks of an item side by side, statistics blocks summed by a second launch
    (dict(kind="rat", D=16, depth=2, R=2), 16, 1, BERNOULLI, 1100),        # nine shares of one chunk each
    (dict(kind="pd", H=6, W=6, deltas=[2]), 24, 1, GAUSSIAN, 520),         # three shares of two, two and one chunk
    # twelve strips: ten layers of 11 to 36 items below the root that all split their nine chunks, more than the eight whose sums the
    # launch at the end of the pass takes; the two bottom layers walk their chunks in turn
    (dict(kind="pd", H=2, W=24, deltas=[2], axes=2), 8, 1, BERNOULLI, 1100),
]


@pytest.mark.parametrize("spec,K,C,family,B", CASES)
def test_einsum_kernels_for_every_tile_shape(spec, K, C, family, B):
    print("einsum shape case", spec, K, C, family, B, flush=True)
    seed = 4000 + K + B
    oracle, flat, rng = make_oracle(spec, K, C, family, seed, leaf_range=(0.1, 0.9))
    D = oracle.g.num_vars
    x = workloads.draw_data(rng, dict(kind="bernoulli_iid", p=0.4) if family == BERNOULLI
                            else dict(kind="gaussian_mixture", components=3, std=0.3), B, D, C)
    m = gpu_model(spec, K, C, family, B, seed, flat)
    ref_stats, ref_logp = oracle.em_accumulate(x, None)
    ref_flat = oracle.stats_to_flat(ref_stats)
    assert_logp_close(m.logp(dev(x)), ref_logp)
    lp = torch.empty(B, device="cuda")
    m.em_accumulate(dev(x), None, lp)
    assert_logp_close(lp, ref_logp)
    assert_stats_close(m.stats, ref_flat, oracle.layout, m.n_params)
    # a second E-step adds to the statistics (the kernels read them back)
    m.em_accumulate(dev(x), None, lp)
    assert_stats_close(m.stats, 2.0 * ref_flat, oracle.layout, m.n_params)
    # after an M-step the einsum-weight statistics are overwritten, not added to
    kw = dict(step=0.5, min_var=1e-4, max_var=2.0, w_floor=1e-9) if family == GAUSSIAN else dict(step=0.5, w_floor=1e-9)
    m.em_update(**kw)
    oracle.em_update(oracle.stats_from_flat(2.0 * ref_flat), **kw)
    ref_p = oracle.get_flat_params()
    got_p = m.params.cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got_p - ref_p) <= 1e-3 * np.abs(ref_p) + 1e-7)
    m.set_params(ref_p)                                  # (both sides continue from the oracle's parameters)
    oracle.set_flat_params(ref_p)
    ref2, ref_logp2 = oracle.em_accumulate(x, None)
    m.em_accumulate(dev(x), None, lp)
    assert_logp_close(lp, ref_logp2)
    assert_stats_close(m.stats, oracle.stats_to_flat(ref2), oracle.layout, m.n_params)
    # a smaller batch on the same handle
    nb = max(1, B // 3)
    m.em_reset()
    m.em_accumulate(dev(x[:nb]), None, lp[:nb])
    ref3, _ = oracle.em_accumulate(x[:nb], None)
    assert_stats_close(m.stats, oracle.stats_to_flat(ref3), oracle.layout, m.n_params)
    m.close()


LONG_SCOPES = [
    # spec, K, C, family, B: leaves with at least 1024 (variable, channel) pairs take the statistics kernel on the matrix
    # pipe when nothing is marginalised
    (dict(kind="rat", D=2500, depth=1, R=2), 5, 1, BERNOULLI, 70),         # one statistic, one column tile, ragged pairs
    (dict(kind="pd", H=48, W=44, deltas=[24]), 33, 3, GAUSSIAN, 130),      # two statistics, two column tiles, three passes
    (dict(kind="pd", H=32, W=40, deltas=[20], axes=2), 8, 1, GAUSSIAN, 64),   # strips of 640 and 640 pixels: below the limit
]


@pytest.mark.parametrize("spec,K,C,family,B", LONG_SCOPES)
def test_leaf_statistics_of_very_long_scopes(spec, K, C, family, B):
    print("long scope case", spec, K, C, family, B, flush=True)
    seed = 5000 + K + B
    oracle, flat, rng = make_oracle(spec, K, C, family, seed, leaf_range=(0.2, 0.8))
    D = oracle.g.num_vars
    x = workloads.draw_data(rng, dict(kind="bernoulli_iid", p=0.4) if family == BERNOULLI
                            else dict(kind="gaussian_mixture", components=3, std=0.3), B, D, C)
    m = gpu_model(spec, K, C, family, B, seed, flat)
    ref_stats, ref_logp = oracle.em_accumulate(x, None)
    ref_flat = oracle.stats_to_flat(ref_stats)
    lp = torch.empty(B, device="cuda")
    m.em_accumulate(dev(x), None, lp)
    assert_logp_close(lp, ref_logp)
    assert_stats_close(m.stats, ref_flat, oracle.layout, m.n_params)
    m.em_accumulate(dev(x), None, lp)                    # added to, not overwritten
    assert_stats_close(m.stats, 2.0 * ref_flat, oracle.layout, m.n_params)
    # with a mask the element-wise kernel runs; both must agree with the oracle
    mask = workloads.draw_mask(rng, dict(kind="shared", observed_fraction=0.7), B, D)
    ref_m, _ = oracle.em_accumulate(x, mask)
    m.em_reset()
    m.em_accumulate(dev(x), dev(mask), lp)
    assert_stats_close(m.stats, oracle.stats_to_flat(ref_m), oracle.layout, m.n_params)
    m.close()


ROOT_CASES = [
    # spec, K, C, family, B: the top of the circuit (the root's partitions and the root's mixture in one launch)
    (dict(kind="rat", D=8, depth=1, R=1), 64, 1, BERNOULLI, 5),            # one partition, no mixture, widest K, B below a tile
    (dict(kind="rat", D=8, depth=1, R=40), 64, 1, BERNOULLI, 33),          # widest K and many partitions: more than 64 KB of LDS
    (dict(kind="rat", D=8, depth=2, R=3), 7, 2, GAUSSIAN, 130),            # K not a multiple of 4
    (dict(kind="rat", D=6, depth=1, R=300), 64, 1, BERNOULLI, 9),          # just within the 160 KB of LDS
    (dict(kind="rat", D=6, depth=1, R=320), 64, 1, BERNOULLI, 9),          # too many partitions for the LDS: general kernels
    (dict(kind="pd", H=4, W=4, deltas=[2]), 1, 1, GAUSSIAN, 70),           # K = 1
]


@pytest.mark.parametrize("spec,K,C,family,B", ROOT_CASES)
def test_root_of_the_circuit(spec, K, C, family, B):
    print("root case", spec, K, C, family, B, flush=True)
    seed = 6000 + K + B
    oracle, flat, rng = make_oracle(spec, K, C, family, seed, leaf_range=(0.1, 0.9))
    D = oracle.g.num_vars
    x = workloads.draw_data(rng, dict(kind="bernoulli_iid", p=0.4) if family == BERNOULLI
                            else dict(kind="gaussian_mixture", components=3, std=0.3), B, D, C)
    m = gpu_model(spec, K, C, family, B, seed, flat)
    ref_stats, ref_logp = oracle.em_accumulate(x, None)
    assert_logp_close(m.logp(dev(x)), ref_logp)
    lp = torch.empty(B, device="cuda")
    m.em_accumulate(dev(x), None, lp)
    assert_logp_close(lp, ref_logp)
    assert_stats_close(m.stats, oracle.stats_to_flat(ref_stats), oracle.layout, m.n_params)
    # a marginalised batch, then a smaller one on the same handle
    mask = workloads.draw_mask(rng, dict(kind="per_sample", observed_fraction=0.5), B, D)
    assert_logp_close(m.logp(dev(x), dev(mask)), oracle.logp(x, mask))
    nb = max(1, B // 2)
    assert_logp_close(m.logp(dev(x[:nb])), ref_logp[:nb])
    m.close()


TREES = [
    # spec, K, C, family, B, mask kind, posterior-assembly launches expected per E-step.  In a random binary tree every
    # region has one partition and one parent partition: the 16x16x4 top-down kernel and the element-wise leaf statistics
    # take the posterior from the parent's blocks, and nothing is assembled by a launch of its own.
    (dict(kind="rat", D=40, depth=3, R=3), 10, 1, BERNOULLI, 100, None, 0),        # K not a multiple of 4, three blocks
    (dict(kind="rat", D=40, depth=3, R=3), 7, 2, GAUSSIAN, 130, "per_sample", 0),  # two chunks of the batch, masks
    (dict(kind="rat", D=64, depth=4, R=2), 20, 1, GAUSSIAN, 96, "shared", 0),      # 16-byte loads, up to five blocks
    (dict(kind="rat", D=300, depth=2, R=8), 12, 1, GAUSSIAN, 70, None, 0),         # leaves of 75 variables: cell form
    (dict(kind="rat", D=12, depth=1, R=3), 5, 1, BERNOULLI, 33, None, 0),          # leaves right under the root
    (dict(kind="rat", D=40, depth=3, R=3), 28, 1, BERNOULLI, 64, None, 3),         # seven blocks per right child: assembled
    (dict(kind="rat", D=40, depth=3, R=3), 16, 1, BERNOULLI, 64, None, 2),         # kernel with specialised waves: inner layers assembled
    (dict(kind="rat", D=40, depth=3, R=3), 6, 1, 3, 50, None, 1),                  # categorical leaves read the assembled posterior
]


@pytest.mark.parametrize("spec,K,C,family,B,mask_kind,assemblies", TREES)
def test_trees_take_posteriors_from_the_parents_blocks(spec, K, C, family, B, mask_kind, assemblies):
    print("tree case", spec, K, C, family, B, mask_kind, flush=True)
    seed = 5100 + K + B
    leaf_param = 4 if family == 3 else 0
    oracle, flat, rng = make_oracle(spec, K, C, family, seed, leaf_range=(0.1, 0.9), leaf_param=leaf_param)
    D = oracle.g.num_vars
    data = (dict(kind="bernoulli_iid", p=0.4) if family == BERNOULLI else
            dict(kind="categorical_mixture", components=3, values=4) if family == 3 else dict(kind="gaussian_mixture", components=3, std=0.3))
    x = workloads.draw_data(rng, data, B, D, C)
    mask = workloads.draw_mask(rng, None if mask_kind is None else dict(kind=mask_kind, observed_fraction=0.7), B, D)
    m = gpu_model(spec, K, C, family, B, seed, flat, leaf_param=leaf_param)
    ref_stats, ref_logp = oracle.em_accumulate(x, mask)
    ref_flat = oracle.stats_to_flat(ref_stats)
    lp = torch.empty(B, device="cuda")
    m.em_accumulate(dev(x), dev(mask), lp)          # (the first E-step also writes the root's ones)
    assert_logp_close(lp, ref_logp)
    assert_stats_close(m.stats, ref_flat, oracle.layout, m.n_params)
    m.profile_enable(True)
    m.em_accumulate(dev(x), dev(mask), lp)          # adds to the statistics
    torch.cuda.synchronize()
    prof = m.profile_read()
    m.profile_enable(False)
    assert_stats_close(m.stats, 2.0 * ref_flat, oracle.layout, m.n_params)
    assert prof.get("region_backward", (0.0, 0))[1] == assemblies, prof
    # a smaller batch on the same handle, statistics overwritten after an M-step
    kw = dict(step=0.5, min_var=1e-4, max_var=2.0, w_floor=1e-9) if family == GAUSSIAN else dict(step=0.5, w_floor=1e-9)
    m.em_update(**kw)
    oracle.em_update(oracle.stats_from_flat(2.0 * ref_flat), **kw)
    m.set_params(oracle.get_flat_params())
    nb = max(1, B // 3)
    m.em_reset()
    mask3 = mask if mask is None or mask.ndim == 1 else mask[:nb]
    m.em_accumulate(dev(x[:nb]), dev(mask3), lp[:nb])
    ref3, ref_logp3 = oracle.em_accumulate(x[:nb], mask3)
    assert_logp_close(lp[:nb], ref_logp3)
    assert_stats_close(m.stats, oracle.stats_to_flat(ref3), oracle.layout, m.n_params)
    m.close()
