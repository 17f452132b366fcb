"""The allocation-free entry point einet_logp_static (activations in the library's fixed device arena) against
einet_logp (activations in the caller's workspace), through the C ABI: same kernels, so the results must agree
bit for bit, on two calls in a row, the second with a smaller batch; and against the oracle to the logP tolerance."""
import ctypes as C

import numpy as np
import pytest
import torch

import paper_2004_06231_amd as P
import workloads
from oracle.einet import GAUSSIAN
from tests.common import make_oracle
from tests.gpu_common import gpu_model, dev, assert_logp_close

pytestmark = pytest.mark.gpu


def _call(lib, fn, m, x, mask, out):
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    mp, mode = (None, P.binding.MASK_NONE) if mask is None else (C.c_void_p(mask.data_ptr()), P.binding.MASK_SHARED)
    rc = fn(m._h, C.c_void_p(x.data_ptr()), mp, mode, x.shape[0], C.c_void_p(out.data_ptr()), stream)
    assert rc == 0, lib.einet_last_error(m._h)


def test_static_arena_logp_matches_workspace_logp_on_two_calls():
    lib = P.load_library()
    spec, K, Cn = dict(kind="pd", H=8, W=8, deltas=[4, 2]), 12, 2
    oracle, flat, rng = make_oracle(spec, K, Cn, GAUSSIAN, 91)
    D = oracle.g.num_vars
    x = workloads.draw_data(rng, dict(kind="gaussian_mixture", components=4, std=0.2), 70, D, Cn)
    mask = workloads.draw_mask(rng, dict(kind="shared", observed_fraction=0.7), 70, D)
    m = gpu_model(spec, K, Cn, GAUSSIAN, 70, 91, flat)
    # first call: 70 samples (several sample tiles and a ragged tail), with a mask; second call: 23 samples, no mask
    for n, msk in ((70, mask), (23, None)):
        print(f"einet_logp_static with {n} samples, mask {'shared' if msk is not None else 'none'}", flush=True)
        xd, md = dev(x[:n]), dev(msk)
        want = torch.full((n,), float("nan"), device="cuda")
        got = torch.full((n,), float("nan"), device="cuda")
        _call(lib, lib.einet_logp, m, xd, md, want)
        _call(lib, lib.einet_logp_static, m, xd, md, got)
        torch.cuda.synchronize()
        assert torch.equal(got, want)
        assert_logp_close(got, oracle.logp(x[:n], msk))
    # the workspace path still works after the arena was used, and the arena after the workspace
    a = m.logp(dev(x)).clone()
    b = torch.empty(70, device="cuda")
    m.logp_static(dev(x), b)
    assert torch.equal(a, b)
    m.close()


def test_static_arena_rejects_what_does_not_fit():
    lib = P.load_library()
    spec, K = dict(kind="rat", D=64, depth=5, R=8), 32
    oracle, flat, rng = make_oracle(spec, K, 1, GAUSSIAN, 92)
    B = 2048                                           # 4 * nodes * B * K alone is far beyond the 16 MiB arena
    m = gpu_model(spec, K, 1, GAUSSIAN, B, 92, flat)
    x = torch.zeros(B, 64, 1, device="cuda")
    out = torch.zeros(B, device="cuda")
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    rc = lib.einet_logp_static(m._h, C.c_void_p(x.data_ptr()), None, 0, B, C.c_void_p(out.data_ptr()), stream)
    assert rc == -4 and b"arena" in lib.einet_last_error(m._h)
    # a batch that fits goes through on the same handle
    small = workloads.draw_data(rng, dict(kind="gaussian_mixture", components=2, std=0.3), 16, 64, 1)
    got = torch.empty(16, device="cuda")
    m.logp_static(dev(small), got)
    assert_logp_close(got, oracle.logp(small))
    m.close()
