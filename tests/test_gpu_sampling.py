"""GPU parity of top-down sampling (einet_sample) against oracle/sampling.py on the same random numbers.

The choices at the sums are integers decided by floating-point sums: the kernels decide them in float32, the
oracle in float64.  With K*K pairs to choose from, the interval of a pair is about 1/K^2 of the total wide
(6e-4 for K = 40), the float32 running sums are good to about 1e-6 of the total, so a small share of the choices
can fall on the other side of a boundary.  Every sample whose choices all stayed at least MARGIN (relative to
the total weight) away from the boundaries of their intervals must agree with the oracle entry by entry; of all
samples at least `min_fraction` must agree; every other sample must be the one the oracle draws when one of its
near-tie choices (margin below MARGIN) falls on the other side of the nearer boundary and the descent continues
from there (`oracle.sampling.sample(..., flip=...)`), besides the validity checks (finite values, evidence kept,
Bernoulli values in {0, 1})."""
import numpy as np
import pytest
import torch

import paper_2004_06231_amd as P
import workloads
from oracle.einet import BERNOULLI, GAUSSIAN
from oracle.sampling import sample
from tests.common import make_oracle, make_config
from tests.gpu_common import gpu_model, dev

pytestmark = pytest.mark.gpu

MARGIN = 1e-5

CASES = [
    # spec, K, C, family, B, evidence, leaf values
    (dict(kind="rat", D=8, depth=3, R=2), 4, 1, BERNOULLI, 64, None, "draw"),
    (dict(kind="rat", D=9, depth=2, R=1), 1, 1, BERNOULLI, 5, None, "draw"),                 # K = 1: nothing to choose
    (dict(kind="rat", D=16, depth=3, R=3), 3, 2, BERNOULLI, 17, "shared", "draw"),
    (dict(kind="rat", D=20, depth=2, R=2), 5, 1, GAUSSIAN, 33, "per_sample", "draw"),
    (dict(kind="rat", D=40, depth=3, R=2), 13, 1, GAUSSIAN, 70, None, "mean"),
    (dict(kind="rat", D=10, depth=2, R=1), 64, 1, BERNOULLI, 20, "shared", "mean"),          # largest K
    (dict(kind="rat", D=64, depth=5, R=2), 64, 1, GAUSSIAN, 9, "per_sample", "draw"),
    (dict(kind="pd", H=6, W=6, deltas=[2]), 6, 3, GAUSSIAN, 19, "shared", "mean"),
    (dict(kind="pd", H=8, W=4, deltas=[4, 2]), 9, 1, BERNOULLI, 40, None, "draw"),
    (dict(kind="pd", H=4, W=12, deltas=[4], axes=2), 17, 2, GAUSSIAN, 200, "per_sample", "draw"),
]


def _compare(oracle, m, B, rng, x, mask, values, family, min_fraction=0.9):
    g = oracle.g
    D, C = g.num_vars, oracle.C
    u = rng.random((g.num_partitions + g.num_regions, B), dtype=np.float32)
    noise = None
    if values == "draw":
        noise = (rng.standard_normal((B, D, C)) if family == GAUSSIAN else rng.random((B, D, C))).astype(np.float32)
    got = m.sample(B, dev(u), dev(noise), dev(x), dev(mask)).cpu().numpy().astype(np.float64)
    ref, margin, _ = sample(oracle, B, u.astype(np.float64), None if noise is None else noise.astype(np.float64),
                            x, mask)
    assert np.all(np.isfinite(got))
    if mask is not None:
        obs = np.broadcast_to(np.asarray(mask, bool) if np.ndim(mask) == 2 else np.asarray(mask, bool)[None], (B, D))
        assert np.array_equal(got[obs], np.asarray(x, np.float64)[obs])            # evidence is kept, bit for bit
    if family == BERNOULLI and values == "draw":
        assert np.all((got == 0.0) | (got == 1.0))
    err = np.abs(got - ref)
    same = np.all(err <= 1e-5 * np.abs(ref) + 1e-6, axis=(1, 2))
    clear = margin >= MARGIN
    assert np.all(same[clear]), f"{int((~same[clear]).sum())} samples with clear-cut choices differ"
    assert same.mean() >= min_fraction, f"only {same.mean():.2f} of the samples agree"
    # a sample that differs took the neighbouring interval at one near-tie: flip the near-ties of its reference
    # descent one at a time until the oracle reproduces it
    u64 = u.astype(np.float64)
    n64 = None if noise is None else noise.astype(np.float64)
    for b in np.nonzero(~same)[0]:
        ok = False
        for j in range(8):
            alt, _, _ = sample(oracle, B, u64, n64, x, mask, only=[int(b)], flip={int(b): j}, tie_margin=MARGIN)
            if np.all(np.abs(got[b] - alt[b]) <= 1e-5 * np.abs(alt[b]) + 1e-6):
                ok = True
                break
        assert ok, f"sample {b} differs from the oracle and from every single near-tie alternative"
    return float(same.mean())


@pytest.mark.parametrize("spec,K,C,family,B,evidence,values", CASES)
def test_samples_match_oracle(spec, K, C, family, B, evidence, values):
    seed = 300 + K + B
    print("sampling case", spec, K, C, family, B, evidence, values, flush=True)
    oracle, flat, rng = make_oracle(spec, K, C, family, seed, leaf_range=(0.15, 0.85))
    D = oracle.g.num_vars
    x = mask = None
    if evidence is not None:
        x = workloads.draw_data(rng, dict(kind="bernoulli_iid", p=0.4) if family == BERNOULLI
                                else dict(kind="gaussian_mixture", components=3, std=0.3), B, D, C)
        mask = workloads.draw_mask(rng, dict(kind=evidence, observed_fraction=0.5), B, D)
    m = gpu_model(spec, K, C, family, B, seed, flat)
    _compare(oracle, m, B, rng, x, mask, values, family)
    # a second call with other numbers on the same handle (the selection table is rebuilt every call)
    _compare(oracle, m, B, rng, x, mask, values, family)
    m.close()


def test_inpainting_on_benchmark_configuration_4():
    """Full-size structure and K (PD 32x32x3, K = 40): the left half of every image is observed, the right half is
    drawn from the conditional, once with leaf samples and once with leaf means."""
    cfg, oracle, flat, x, _ = make_config(4, batch=24)
    m = gpu_model(cfg["structure"], cfg["K"], cfg["channels"], cfg["family"], 24, workloads.config_seed(4), flat)
    mask = np.zeros((32, 32), dtype=np.uint8)
    mask[:, :16] = 1
    rng = np.random.default_rng(4)
    for values in ("draw", "mean"):
        print("inpainting", values, flush=True)
        _compare(oracle, m, 24, rng, x, mask.ravel(), values, GAUSSIAN, min_fraction=0.8)
    m.close()


def test_unconditional_samples_of_the_sec42_component_shape():
    cfg = workloads.sec42_config("svhn")
    oracle, flat, rng = make_oracle(cfg["structure"], cfg["K"], 3, GAUSSIAN, 77, cfg["leaf_range"])
    m = gpu_model(cfg["structure"], cfg["K"], 3, GAUSSIAN, 48, 77, flat)
    _compare(oracle, m, 48, rng, None, None, "mean", GAUSSIAN)
    m.close()


def test_sampling_leaves_the_statistics_alone_and_rejects_bad_arguments():
    spec = dict(kind="rat", D=8, depth=2, R=2)
    oracle, flat, rng = make_oracle(spec, 3, 1, BERNOULLI, 5)
    m = gpu_model(spec, 3, 1, BERNOULLI, 16, 5, flat)
    x = dev(workloads.draw_data(rng, dict(kind="bernoulli_iid", p=0.5), 16, 8, 1))
    m.em_accumulate(x)
    before = m.stats.clone()
    n = oracle.g.num_partitions + oracle.g.num_regions
    u = torch.rand(n, 16, device="cuda")
    m.sample(16, u, None)
    assert torch.equal(before, m.stats)
    lib = P.load_library()
    out = torch.empty(16, 8, 1, device="cuda")
    # evidence without a mask, a mask without evidence, too many samples, missing uniforms
    assert lib.einet_sample(m._h, 16, x.data_ptr(), None, 0, u.data_ptr(), None, out.data_ptr(), None) < 0
    assert lib.einet_sample(m._h, 16, None, None, 1, u.data_ptr(), None, out.data_ptr(), None) < 0
    assert lib.einet_sample(m._h, 17, None, None, 0, u.data_ptr(), None, out.data_ptr(), None) < 0
    assert lib.einet_sample(m._h, 16, None, None, 0, None, None, out.data_ptr(), None) < 0
    m.close()
