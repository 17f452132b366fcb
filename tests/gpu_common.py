"""Helpers for the GPU parity tests: build the HIP model next to the oracle model."""
import numpy as np
import torch

import paper_2004_06231_amd as P
from tests.common import make_config, make_oracle

LOGP_RTOL, LOGP_ATOL = 1e-4, 1e-5       # |d| <= 1e-4 |ref| + 1e-5
STAT_RTOL, STAT_ATOL_REL = 1e-3, 1e-6   # per tensor: |d| <= 1e-3 |ref| + 1e-6 max|ref|


def gpu_model(spec, K, channels, family, max_batch, seed, flat, leaf_param=0):
    m = P.EiNet(spec, K, channels, family, max_batch, seed, leaf_param).bind("cuda:0")
    m.set_params(flat)
    return m


def gpu_config(i, batch=None):
    cfg, oracle, flat, x, mask = make_config(i, batch)
    m = gpu_model(cfg["structure"], cfg["K"], cfg["channels"], cfg["family"], x.shape[0],
                  __import__("workloads").config_seed(i), flat)
    return cfg, oracle, m, flat, x, mask


def dev(a):
    return None if a is None else torch.as_tensor(np.ascontiguousarray(a)).cuda()


def assert_logp_close(got, ref):
    got = got.detach().cpu().numpy().astype(np.float64) if torch.is_tensor(got) else np.asarray(got, np.float64)
    err = np.abs(got - ref)
    tol = LOGP_RTOL * np.abs(ref) + LOGP_ATOL
    assert np.all(np.isfinite(got)), "non-finite logP"
    assert np.all(err <= tol), f"logP: worst |d|={err.max():.3e} at ref={ref[err.argmax()]:.6f}, tol={tol[err.argmax()]:.3e}"
    return float((err / np.abs(ref).clip(1e-30)).max())


def stat_tensors(flat, lay, n_params):
    """Split a flat statistics vector into the tensors the tolerance is stated for."""
    first_v = min(lay.v_off.values()) if lay.v_off else lay.phi_off
    return {"Nw": flat[:first_v], "Nv": flat[first_v:lay.phi_off], "num": flat[lay.phi_off:n_params],
            "den": flat[lay.den_off:lay.tot_off], "tot": flat[lay.tot_off:]}


def assert_stats_close(got_flat, ref_flat, lay, n_params, rtol=STAT_RTOL, atol_rel=STAT_ATOL_REL):
    got_flat = got_flat.detach().cpu().numpy().astype(np.float64) if torch.is_tensor(got_flat) else got_flat
    worst = {}
    g, r = stat_tensors(got_flat, lay, n_params), stat_tensors(ref_flat, lay, n_params)
    for name in r:
        if r[name].size == 0:
            continue
        err = np.abs(g[name] - r[name])
        tol = rtol * np.abs(r[name]) + atol_rel * np.abs(r[name]).max()
        assert np.all(np.isfinite(g[name])), name
        i = int((err - tol).argmax())
        assert np.all(err <= tol), f"{name}: |d|={err[i]:.3e} ref={r[name][i]:.6e} tol={tol[i]:.3e} at {i}"
        scale = np.abs(r[name]) + atol_rel * np.abs(r[name]).max() / rtol
        worst[name] = float((err[scale > 0] / scale[scale > 0]).max()) if np.any(scale > 0) else 0.0
    return worst
