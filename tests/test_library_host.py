"""Host-side checks of libeinet.so that need no GPU: the library loads, exports every
symbol the header declares, rejects bad arguments, and its structure compiler builds,
integer for integer, the graph, layers and parameter layout the oracle builds on its own."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2004_06231_amd as P
from oracle import structure as S
from tests.common import oracle_graph
import workloads

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "einet.h")).read()
    declared = set(re.findall(r"\b(einet_[a-z_]+)\s*\(", header))
    assert declared == set(P.EXPORTED_SYMBOLS)
    lib = ctypes.CDLL(P.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name


SPECS = [
    (dict(kind="rat", D=8, depth=3, R=2), 4, 1, 11),
    (dict(kind="rat", D=784, depth=8, R=10), 10, 1, workloads.config_seed(2)),
    (dict(kind="rat", D=37, depth=4, R=1), 3, 2, 2 ** 63 + 5),
    (dict(kind="pd", H=28, W=28, deltas=[7]), 16, 1, 0),
    (dict(kind="pd", H=32, W=32, deltas=[8]), 40, 3, 0),
    (dict(kind="pd", H=64, W=64, deltas=[16, 8]), 20, 3, 0),
    (dict(kind="pd", H=32, W=32, deltas=[8], axes=2), 5, 3, 0),
    (dict(kind="pd", H=5, W=7, deltas=[3, 2, 1]), 2, 1, 0),
]


@pytest.mark.parametrize("spec,K,C,seed", SPECS)
def test_structure_matches_oracle(spec, K, C, seed):
    family = P.GAUSSIAN
    m = P.EiNet(spec, K, C, family, max_batch=4, seed=seed)
    st = m.structure()
    g = oracle_graph(spec, seed)
    assert (st["num_vars"], st["num_regions"], st["num_partitions"], st["num_replica"]) == \
        (g.num_vars, g.num_regions, g.num_partitions, g.num_replica)
    for s in range(g.num_regions):
        assert tuple(st["scope_var"][st["scope_ptr"][s]:st["scope_ptr"][s + 1]]) == g.scopes[s]
    assert [tuple(p) for p in st["partition"]] == list(g.partitions)
    assert list(st["region_replica"]) == list(g.replica)
    # Algorithm 1 layers
    _, prod_layers = S.topological_layers(g)
    assert st["num_layers"] == len(prod_layers)
    for l, layer in enumerate(prod_layers):
        assert list(st["layer_partition"][st["layer_ptr"][l]:st["layer_ptr"][l + 1]]) == layer
    # parameter / statistics layout
    lay = S.param_layout(g, K, C, 2)
    assert list(st["w_offset"]) == lay.w_off
    assert {s: int(o) for s, o in enumerate(st["v_offset"]) if o >= 0} == lay.v_off
    assert (st["phi_offset"], st["den_offset"], st["tot_offset"]) == (lay.phi_off, lay.den_off, lay.tot_off)
    assert (m.n_params, m.n_stats) == (lay.n_params, lay.n_stats)
    m.close()


def test_create_rejects_bad_arguments():
    ok = dict(kind="rat", D=8, depth=2, R=1)
    for bad, code in [
        ((dict(kind="rat", D=4, depth=3, R=1), 4, 1, 0, 8), -2),       # one-variable scope would split
        ((dict(kind="pd", H=8, W=8, deltas=[8]), 4, 1, 0, 8), -2),      # no cut
        ((ok, 0, 1, 0, 8), -1), ((ok, 65, 1, 0, 8), -1), ((ok, 4, 0, 0, 8), -1),
        ((ok, 4, 1, 7, 8), -1), ((ok, 4, 1, 0, 0), -1),
        ((dict(kind="rat", D=8, depth=0, R=1), 4, 1, 0, 8), -1),
        ((dict(kind="pd", H=8, W=8, deltas=[]), 4, 1, 0, 8), -1),
        ((dict(kind="pd", H=8, W=8, deltas=[4], axes=0), 4, 1, 0, 8), -1),
    ]:
        with pytest.raises(P.EinetError) as e:
            P.EiNet(*bad)
        assert e.value.code == code
        assert len(str(e.value)) > 20


def test_calls_before_bind_fail_cleanly():
    m = P.EiNet(dict(kind="rat", D=8, depth=2, R=1), 4, 1, 0, 8)
    lib = P.load_library()
    assert lib.einet_refresh(m._h, None) == -3
    assert lib.einet_em_update(m._h, 1.0, 0.0, 1.0, 0.0, None) == -3
    assert lib.einet_em_reset(m._h, None) == -3
    assert lib.einet_logp(m._h, None, None, 0, 4, None, None) == -3
    assert lib.einet_bind(m._h, None, None, None, None) == -1
    assert b"NULL" in lib.einet_last_error(m._h)
    assert lib.einet_sizes(None, None, None, None) == -1
    with pytest.raises(RuntimeError):
        import torch
        if torch.cuda.is_available():
            raise RuntimeError("GPU present: bind would succeed")
        m.bind()


def test_bench_refuses_more_than_one_gpu():
    """This build runs on one GPU; bench.py says so and exits before it touches a device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr
    assert r.stdout.strip() == ""
