"""Helpers shared by the tests: build the oracle model of a workload."""
import numpy as np

from oracle import structure as ostruct
from oracle.einet import OracleEiNet, num_stats
import workloads


def oracle_graph(spec, seed):
    if spec["kind"] == "rat":
        return ostruct.rat_structure(spec["D"], spec["depth"], spec["R"], seed)
    return ostruct.pd_structure(spec["H"], spec["W"], spec["deltas"], spec.get("axes", 3))


def weight_blocks_of(graph, K, layout):
    blocks = []
    for n, (parent, _, _) in enumerate(graph.partitions):
        blocks.append((layout.w_off[n], graph.k_out(parent, K), K * K))
    for s, off in layout.v_off.items():
        blocks.append((off, graph.k_out(s, K), len(graph.children[s])))
    return blocks


def make_oracle(spec, K, channels, family, seed, leaf_range=(0.1, 0.9), rng=None, leaf_param=0):
    """Oracle model with Dirichlet(1) weights and uniform leaf parameters.
    Returns (model, flat float32 parameters, rng)."""
    g = oracle_graph(spec, seed)
    model = OracleEiNet(g, K, channels, family, leaf_param)
    lay = model.layout
    if rng is None:
        rng = np.random.default_rng(seed)
    T = num_stats(family, leaf_param)
    flat = workloads.draw_params(
        rng, lay.n_params, weight_blocks_of(g, K, lay), lay.phi_off,
        (g.num_vars, channels, g.num_replica, T, K), family, leaf_range, leaf_param)
    model.set_flat_params(flat)
    return model, flat, rng


def make_config(i, batch=None):
    """Oracle model + inputs of benchmark configuration i (1-based)."""
    cfg = workloads.get_config(i)
    seed = workloads.config_seed(i)
    model, flat, rng = make_oracle(cfg["structure"], cfg["K"], cfg["channels"], cfg["family"],
                                   seed, cfg["leaf_range"])
    B = cfg["B"] if batch is None else batch
    D = model.g.num_vars
    x = workloads.draw_data(rng, cfg["data"], B, D, cfg["channels"])
    mask = workloads.draw_mask(rng, cfg["mask"], B, D)
    return cfg, model, flat, x, mask


def all_binary(D):
    """[2^D, D, 1] array of every binary assignment."""
    idx = np.arange(2 ** D)
    return ((idx[:, None] >> np.arange(D)[None, :]) & 1).astype(np.float64)[:, :, None]


def normalise_exactly(model):
    """float32-rounded rows sum to 1 only to 1e-7; make them exact in float64."""
    for n in range(len(model.W)):
        model.W[n] /= model.W[n].sum(axis=(1, 2), keepdims=True)
    for s in model.v:
        model.v[s] /= model.v[s].sum(axis=1, keepdims=True)
