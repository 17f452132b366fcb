"""An epoch of stochastic EM (Sec. 3.5: E-step and M-step per mini-batch) captured into a HIP graph and replayed:
every replay must leave exactly what the same epoch leaves when its launches are enqueued one by one.  The replays
alternate with eager work on the same handle and with synchronisations, as a training loop's would."""
import numpy as np
import pytest
import torch

import paper_2004_06231_amd as P
import workloads
from oracle.einet import BERNOULLI, GAUSSIAN

pytestmark = pytest.mark.gpu

CASES = [
    # spec, K, C, family, batch, N: the last mini-batch is ragged in both
    (dict(kind="pd", H=8, W=8, deltas=[4]), 8, 1, GAUSSIAN, 64, 200),
    (dict(kind="rat", D=24, depth=2, R=3), 40, 1, BERNOULLI, 300, 700),     # several chunks per mini-batch: virtual items
]


@pytest.mark.parametrize("spec,K,C,family,batch,N", CASES)
def test_replayed_epoch_equals_eager_epoch(spec, K, C, family, batch, N):
    print("graph replay case", spec, K, C, family, batch, N, flush=True)
    rng = np.random.default_rng(11)
    eager = P.EiNet(spec, K, C, family, batch, 5).bind("cuda:0")
    graph = P.EiNet(spec, K, C, family, batch, 5).bind("cuda:0")
    D = int(eager.structure()["num_vars"])
    kind = dict(kind="bernoulli_iid", p=0.4) if family == BERNOULLI else dict(kind="gaussian_mixture", components=3, std=0.3)
    x = torch.as_tensor(workloads.draw_data(rng, kind, N, D, C)).cuda()
    em = dict(step=0.5, w_floor=1e-9)
    if family == GAUSSIAN:
        em.update(min_var=1e-4, max_var=1.0)
    lp_e = torch.empty(N, device="cuda")
    lp_g = torch.empty(N, device="cuda")
    for m in (eager, graph):
        m.init_params(7, 0.2, 0.8)
    eager.em_epoch(x, None, batch=batch, logp=lp_e, **em)          # first epoch on both, launch by launch
    graph.em_epoch(x, None, batch=batch, logp=lp_g, **em)
    torch.cuda.synchronize()
    assert torch.equal(eager.params, graph.params)
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        graph.em_epoch(x, None, batch=batch, logp=lp_g, **em)
    torch.cuda.synchronize()
    for rep in range(3):
        eager.em_epoch(x, None, batch=batch, logp=lp_e, **em)
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(eager.params, graph.params), f"replay {rep}: parameters differ"
        assert torch.equal(lp_e, lp_g), f"replay {rep}: logP differs"
        # eager work on the replayed handle between replays: a forward pass does not disturb what the graph relies on
        a = graph.logp(x[:batch])
        b = eager.logp(x[:batch])
        torch.cuda.synchronize()
        assert torch.equal(a, b)
    assert bool(torch.isfinite(graph.params).all())
    eager.close()
    graph.close()
