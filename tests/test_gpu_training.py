"""GPU parity of what sits around one EM step: the stochastic-EM loop over mini-batches (Eq. 8-9 with the
schedule of Sec. 4.2) and the mixture of several EiNets (Sec. 4.2), against oracle/train.py."""
import numpy as np
import pytest
import torch

import paper_2004_06231_amd as P
import workloads
from oracle.einet import BERNOULLI, GAUSSIAN
from oracle.train import em_epoch, mixture_logp
from tests.common import make_oracle
from tests.gpu_common import gpu_model, dev, assert_logp_close

pytestmark = pytest.mark.gpu

EPOCH_CASES = [
    # spec, K, C, family, batch, N, mask kind
    (dict(kind="rat", D=16, depth=2, R=3), 5, 1, GAUSSIAN, 32, 103, None),            # ragged last mini-batch
    (dict(kind="pd", H=8, W=4, deltas=[4, 2]), 6, 1, BERNOULLI, 40, 120, "per_sample"),
    (dict(kind="pd", H=4, W=8, deltas=[2], axes=2), 12, 3, GAUSSIAN, 150, 450, "shared"),  # mini-batch above 128
    (dict(kind="rat", D=12, depth=2, R=2), 3, 1, BERNOULLI, 50, 20, None),            # fewer samples than one batch
]


def _data(rng, family, N, D, C):
    spec = dict(kind="bernoulli_mixture", components=4, lo=0.1, hi=0.9) if family == BERNOULLI \
        else dict(kind="gaussian_mixture", components=4, std=0.2)
    return workloads.draw_data(rng, spec, N, D, C)


@pytest.mark.parametrize("spec,K,C,family,batch,N,mask_kind", EPOCH_CASES)
def test_epoch_matches_oracle(spec, K, C, family, batch, N, mask_kind):
    seed = 77 + K
    oracle, flat, rng = make_oracle(spec, K, C, family, seed, leaf_range=(0.2, 0.8))
    D = oracle.g.num_vars
    x = _data(rng, family, N, D, C)
    mask = workloads.draw_mask(rng, None if mask_kind is None else dict(kind=mask_kind, observed_fraction=0.7), N, D)
    kw = dict(step=0.5, min_var=1e-4, max_var=0.5, w_floor=1e-9)
    print("epoch case", spec, K, family, batch, N, mask_kind, flush=True)
    m = gpu_model(spec, K, C, family, batch, seed, flat)
    lp = torch.full((N,), float("nan"), device="cuda")
    m.em_epoch(dev(x), dev(mask), batch=batch, logp=lp, **kw)
    ref_lp = em_epoch(oracle, x, mask, batch=batch, **kw)
    assert_logp_close(lp, ref_lp)
    got, ref = m.params.cpu().numpy().astype(np.float64), oracle.get_flat_params()
    err = np.abs(got - ref)
    # one update meets 1e-3 |ref| + 1e-7; the later mini-batches see parameters that already differ by that much
    tol = 2e-3 * np.abs(ref) + 1e-6
    assert np.all(err <= tol), f"worst excess {np.max(err - tol):.3e}"
    # the refreshed leaf constants belong to the final parameters
    assert_logp_close(m.logp(dev(x[:batch]), dev(mask if mask is None or mask.ndim == 1 else mask[:batch])),
                      oracle.logp(x[:batch], mask if mask is None or mask.ndim == 1 else mask[:batch]))
    # the loop in the library is the composition of the two calls, bit for bit
    m2 = gpu_model(spec, K, C, family, batch, seed, flat)
    xd, md = dev(x), dev(mask)
    for b0 in range(0, N, batch):
        mb = md if md is None or md.dim() == 1 else md[b0:b0 + batch].contiguous()
        m2.em_accumulate(xd[b0:b0 + batch].contiguous(), mb)
        m2.em_update(**kw)
    assert torch.equal(m.params, m2.params)
    m.close()
    m2.close()


def test_epoch_rejects_bad_arguments_before_touching_the_parameters():
    spec = dict(kind="rat", D=8, depth=2, R=2)
    oracle, flat, rng = make_oracle(spec, 3, 1, BERNOULLI, 5)
    m = gpu_model(spec, 3, 1, BERNOULLI, 16, 5, flat)
    x = dev(_data(rng, BERNOULLI, 40, 8, 1))
    before = m.params.clone()
    with pytest.raises(P.EinetError):
        m.em_epoch(x, None, batch=17)                  # above max_batch
    with pytest.raises(P.EinetError):
        m.em_epoch(x, None, batch=16, step=0.0)
    with pytest.raises(P.EinetError):
        m.em_epoch(x, None, batch=16, min_var=2.0, max_var=1.0)
    with pytest.raises(P.EinetError):
        m.em_epoch(x[:0], None, batch=16)
    torch.cuda.synchronize()
    assert torch.equal(before, m.params)
    m.close()


def test_second_update_without_statistics_keeps_every_parameter():
    """After an M-step the statistics are zero, so another one has nothing to move (rows and leaves
    without posterior mass keep their parameters)."""
    spec = dict(kind="pd", H=4, W=4, deltas=[2])
    oracle, flat, rng = make_oracle(spec, 4, 1, GAUSSIAN, 9)
    m = gpu_model(spec, 4, 1, GAUSSIAN, 30, 9, flat)
    x = _data(rng, GAUSSIAN, 30, 16, 1)
    m.em_accumulate(dev(x))
    m.em_update(step=0.5)
    once = m.params.clone()
    m.em_update(step=0.5)
    np.testing.assert_allclose(m.params.cpu().numpy(), once.cpu().numpy(), rtol=2e-7, atol=0)
    stats, _ = oracle.em_accumulate(x)
    oracle.em_update(stats, step=0.5)
    oracle.em_update(oracle.zero_stats(), step=0.5)
    ref = oracle.get_flat_params()
    assert np.all(np.abs(m.params.cpu().numpy() - ref) <= 1e-3 * np.abs(ref) + 1e-7)
    m.close()


@pytest.mark.parametrize("n_components,B", [(1, 5), (7, 300), (100, 1000)])
def test_mixture_logp_matches_oracle(n_components, B):
    rng = np.random.default_rng(n_components)
    lp = rng.normal(-700.0, 40.0, size=(n_components, B)).astype(np.float32)
    coef = rng.dirichlet(np.ones(n_components))
    if n_components > 1:
        lp[0, : B // 3] = -np.inf                      # a component that excludes some samples
        lp[:, 1] = -np.inf                             # a sample every component excludes
    log_coef = np.log(coef).astype(np.float32)
    got = P.einet_mixture_logp(dev(lp), dev(log_coef)).cpu().numpy().astype(np.float64)
    ref = mixture_logp(lp.astype(np.float64), log_coef.astype(np.float64))
    fin = np.isfinite(ref)
    assert np.array_equal(np.isneginf(got), np.isneginf(ref))
    assert np.all(np.abs(got[fin] - ref[fin]) <= 1e-4 * np.abs(ref[fin]) + 1e-5)


def test_mixture_of_three_einets_matches_oracle():
    spec = dict(kind="rat", D=24, depth=3, R=2)
    rng = np.random.default_rng(31)
    x = _data(rng, GAUSSIAN, 64, 24, 1)
    rows, ref_rows = [], []
    for seed in (41, 42, 43):
        oracle, flat, _ = make_oracle(spec, 6, 1, GAUSSIAN, seed, leaf_range=(0.2, 0.8))
        m = gpu_model(spec, 6, 1, GAUSSIAN, 64, seed, flat)
        rows.append(m.logp(dev(x)).clone())
        ref_rows.append(oracle.logp(x))
        m.close()
    coef = np.array([0.5, 0.3, 0.2])
    got = P.einet_mixture_logp(torch.stack(rows).contiguous(), dev(np.log(coef).astype(np.float32)))
    assert_logp_close(got, mixture_logp(np.stack(ref_rows), np.log(coef)))


def test_mixture_logp_rejects_bad_arguments():
    lib = P.load_library()
    assert lib.einet_mixture_logp(None, None, 1, 1, None, None) < 0
    assert b"NULL" in lib.einet_last_error(None)
    t = torch.zeros(4, device="cuda")
    assert lib.einet_mixture_logp(t.data_ptr(), t.data_ptr(), 0, 4, t.data_ptr(), None) < 0


@pytest.mark.parametrize("shape,B", [("svhn", 500), ("celeba", 40)])
def test_sec42_component_shapes_match_oracle(shape, B):
    """The mixture component of the image experiments (vertical splits only, four strips, K = 40, RGB Gaussian
    leaves): one E-step and one stochastic update at the paper's settings."""
    from tests.gpu_common import assert_stats_close
    cfg = workloads.sec42_config(shape)
    seed = 4200 + B
    print("sec42 shape", cfg["name"], "B", B, flush=True)
    oracle, flat, rng = make_oracle(cfg["structure"], cfg["K"], 3, GAUSSIAN, seed, cfg["leaf_range"])
    x = workloads.draw_data(rng, cfg["data"], B, oracle.g.num_vars, 3)
    m = gpu_model(cfg["structure"], cfg["K"], 3, GAUSSIAN, B, seed, flat)
    ref_stats, ref_logp = oracle.em_accumulate(x, None, chunk=10)
    lp = torch.empty(B, device="cuda")
    m.em_accumulate(dev(x), None, lp)
    assert_logp_close(lp, ref_logp)
    # log-densities of 5e4 in magnitude (128x128x3): the arena keeps float32 residuals against float64 offsets
    # per (node, sample), so the posteriors do not inherit the resolution of a float32 at that magnitude
    # (6e-3); the statistics are asked to be ten times closer than the usual tolerance here
    rtol = 1e-4
    assert_stats_close(m.stats, oracle.stats_to_flat(ref_stats), oracle.layout, m.n_params, rtol=rtol)
    got_lp = lp.cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got_lp - ref_logp) <= 2e-7 * np.abs(ref_logp))     # float32 rounding of the output
    m.em_update(**cfg["em"])
    oracle.em_update(ref_stats, **cfg["em"])
    ref = oracle.get_flat_params()
    got = m.params.cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got - ref) <= 1e-3 * np.abs(ref) + 1e-7)
    m.close()


@pytest.mark.parametrize("family,param", [(BERNOULLI, 0), (GAUSSIAN, 0), (2, 9), (3, 6)])
def test_init_params_matches_the_oracle_generator(family, param):
    """The library's random initialisation is counter-based; the oracle reproduces the numbers from the seed."""
    from oracle.init import init_params
    spec = dict(kind="pd", H=4, W=6, deltas=[2])
    oracle, flat, _ = make_oracle(spec, 7, 2, family, 3, leaf_param=param)
    m = gpu_model(spec, 7, 2, family, 8, 3, flat, param)
    m.init_params(seed=2 ** 63 + 12345, leaf_lo=0.25, leaf_hi=0.75)
    ref = init_params(oracle, 2 ** 63 + 12345, 0.25, 0.75)
    got = m.params.cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got - ref) <= 2e-6 * np.abs(ref) + 1e-12)
    # the derived leaf constants were refreshed: logP under the new parameters
    oracle.set_flat_params(got)
    rng = np.random.default_rng(0)
    x = rng.integers(0, 2 if family == BERNOULLI else max(param, 2), size=(8, 24, 2)).astype(np.float32)
    assert_logp_close(m.logp(dev(x)), oracle.logp(x))
    with pytest.raises(P.EinetError):
        m.init_params(seed=1, leaf_lo=0.9, leaf_hi=0.1)
    m.close()


def test_statistics_do_not_depend_on_earlier_calls_of_the_handle():
    """The top-down pass keeps the posterior of the root (all ones) in its arena between calls when it can; batch
    sizes going up and down and a sampling call in between (it uses the same arena) must not show in the result."""
    spec = dict(kind="pd", H=4, W=4, deltas=[2, 1])
    K, C, family, seed = 6, 1, GAUSSIAN, 9
    oracle, flat, rng = make_oracle(spec, K, C, family, seed, leaf_range=(0.2, 0.8))
    D = oracle.g.num_vars
    m = gpu_model(spec, K, C, family, 64, seed, flat)
    n_choices = m.structure()["num_partitions"] + m.structure()["num_regions"]
    for step, B in enumerate([40, 17, 40, 64, 3, 64]):
        x = _data(rng, family, B, D, C)
        if step == 3:
            m.sample(8, torch.rand(n_choices, 8, device="cuda"), None)
        fresh = gpu_model(spec, K, C, family, 64, seed, flat)
        m.em_reset()
        fresh.em_reset()
        lp, lp2 = torch.empty(B, device="cuda"), torch.empty(B, device="cuda")
        m.em_accumulate(dev(x), None, lp)
        fresh.em_accumulate(dev(x), None, lp2)
        assert torch.equal(lp, lp2)
        assert torch.equal(m.stats, fresh.stats), f"call {step} with {B} samples"
        ref_stats, _ = oracle.em_accumulate(x, None)
        from tests.gpu_common import assert_stats_close
        assert_stats_close(m.stats, oracle.stats_to_flat(ref_stats), oracle.layout, m.n_params)
        fresh.close()
    m.close()
