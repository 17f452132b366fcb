"""Pins for the oracle's structure code: published generator vectors, the
paper's parameter counts, and the structural properties the paper requires."""
import itertools
import os

import numpy as np
import pytest

from oracle import structure as S


def test_splitmix64_published_vectors():
    # first outputs for seeds 0 and 1234567 as printed with the reference C code of the generator
    r = S.SplitMix64(0)
    assert [r.next() for _ in range(3)] == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]
    r = S.SplitMix64(1234567)
    assert [r.next() for _ in range(3)] == [6457827717110365317, 3203168211198807973, 9817491932198370423]


def _printed_counts():
    """The rounded counts of the caption of Fig. 3, from tests/golden/fig3_parameter_counts.txt."""
    path = os.path.join(os.path.dirname(__file__), "golden", "fig3_parameter_counts.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    return {tuple(int(v) for v in r[:4]): float(r[4]) for r in rows}


# exact counts of this layout for the six models whose rounded counts the caption prints
@pytest.mark.parametrize("args,exact", [
    ((512, 4, 10, 1), 10_400), ((512, 4, 10, 40), 9_385_610), ((512, 1, 10, 10), 103_410),
    ((512, 9, 10, 10), 5_203_410), ((512, 4, 1, 10), 24_340), ((512, 4, 40, 10), 973_640),
])
def test_parameter_counts_of_fig3(args, exact):
    D, depth, R, K = args
    printed = _printed_counts()[args]
    g = S.rat_structure(D, depth, R, seed=3)
    n = S.param_layout(g, K, 1, 2).n_params
    assert abs(n - printed) / printed < 0.05          # the caption's rounded figure
    assert n == exact
    # closed form: R trees of (2^depth - 2) inner partitions with K^3 weights and one root
    # partition with K^2, R root mixing weights (none if R = 1), 2 parameters per (d, k, r)
    assert n == R * ((2 ** depth - 2) * K ** 3 + K ** 2) + (R if R > 1 else 0) + D * K * R * 2


def check_valid(g):
    """Smoothness and decomposability (Sec. 2) in region-graph form."""
    for (parent, left, right) in g.partitions:
        a, b = set(g.scopes[left]), set(g.scopes[right])
        assert a and b and not (a & b)                       # decomposable
        assert a | b == set(g.scopes[parent])                # all partitions of a region share its scope
    assert set(g.scopes[0]) == set(range(g.num_vars))
    # every region except the root is the child of some partition, and every partition has one parent region
    child_of = {c for (_, l, r) in g.partitions for c in (l, r)}
    assert child_of == set(range(1, g.num_regions))
    # replica: leaves with equal replica are disjoint (Sec. 3.4)
    for r in range(g.num_replica):
        seen = set()
        for s in g.leaves():
            if g.replica[s] == r:
                assert not (seen & set(g.scopes[s]))
                seen |= set(g.scopes[s])
    for s in range(g.num_regions):
        assert (g.replica[s] >= 0) == g.is_leaf(s)
        assert list(g.scopes[s]) == sorted(g.scopes[s])


@pytest.mark.parametrize("D,depth,R", [(8, 3, 2), (13, 2, 3), (784, 8, 10), (512, 9, 2)])
def test_rat_is_balanced_binary_tree(D, depth, R):
    g = S.rat_structure(D, depth, R, seed=11)
    check_valid(g)
    assert len(g.leaves()) == R * 2 ** depth
    assert g.num_partitions == R * (2 ** depth - 1)
    assert len(g.children[0]) == R
    for (parent, left, right) in g.partitions:
        assert len(g.scopes[right]) - len(g.scopes[left]) in (0, 1)
    # within a replica the leaves partition the variables
    for r in range(R):
        cover = sorted(v for s in g.leaves() if g.replica[s] == r for v in g.scopes[s])
        assert cover == list(range(D))
    # different replicas / seeds give different trees
    g2 = S.rat_structure(D, depth, R, seed=12)
    assert g.scopes != g2.scopes
    if R > 1:
        assert g.scopes[1] != g.scopes[1 + (2 ** (depth + 1) - 2)]


def test_rat_split_is_a_uniform_shuffle():
    # every variable lands left about half the time over many (replica, node) keys
    n, trials = 10, 4000
    left_count = np.zeros(n)
    for h in range(trials):
        left, right = S.rat_split(tuple(range(n)), seed=99, r=h % 7, h=h + 1)
        assert len(left) == 5 and sorted(left + right) == list(range(n))
        left_count[list(left)] += 1
    assert np.all(np.abs(left_count / trials - 0.5) < 0.04)


def test_rat_errors():
    with pytest.raises(ValueError):
        S.rat_structure(4, 3, 1, 0)       # 4 variables cannot be split to depth 3
    with pytest.raises(ValueError):
        S.rat_structure(8, 0, 1, 0)


def brute_force_pd(H, W, delta, axes=3):
    """Independent enumeration: the set of rectangles reachable from the image by grid cuts."""
    rects, parts = set(), set()
    todo = [(0, H, 0, W)]
    while todo:
        r = todo.pop()
        if r in rects:
            continue
        rects.add(r)
        y0, y1, x0, x1 = r
        if axes & 1:
            for c in range(y0 + delta, y1, delta):
                parts.add((r, "y", c))
                todo += [(y0, c, x0, x1), (c, y1, x0, x1)]
        if axes & 2:
            for c in range(x0 + delta, x1, delta):
                parts.add((r, "x", c))
                todo += [(y0, y1, x0, c), (y0, y1, c, x1)]
    return rects, parts


@pytest.mark.parametrize("H,W,deltas,axes", [(28, 28, [7], 3), (32, 32, [8], 3), (8, 12, [4], 3),
                                            (32, 32, [8], 2), (5, 7, [2], 3)])
def test_pd_matches_rectangle_enumeration(H, W, deltas, axes):
    g = S.pd_structure(H, W, deltas, axes)
    check_valid(g)
    rects, parts = brute_force_pd(H, W, deltas[0], axes)
    assert set(g.rects) == rects and len(g.rects) == len(rects)
    assert g.num_partitions == len(parts)


def test_pd_counts_of_the_benchmark_grids():
    # an n x n grid of cells has C(n+1,2)^2 rectangles; a rectangle of a x b cells has (a-1)+(b-1) cuts
    g = S.pd_structure(32, 32, [8])
    assert (g.num_regions, g.num_partitions, len(g.leaves()), g.num_replica) == (100, 200, 16, 1)
    n_cuts = sum((a - 1) + (b - 1) for a in range(1, 5) for b in range(1, 5) for _ in range((5 - a) * (5 - b)))
    assert n_cuts == 200
    g = S.pd_structure(64, 64, [16, 8])
    assert (g.num_regions, g.num_partitions, len(g.leaves()), g.num_replica) == (228, 296, 64, 1)
    assert all(len(g.scopes[s]) == 64 for s in g.leaves())
    # the coarse step is used while it cuts; the fine one only inside 16x16 cells
    for s, (y0, y1, x0, x1) in enumerate(g.rects):
        if (y1 - y0, x1 - x0) == (16, 16):
            assert len(g.children[s]) == 2
    # vertical-only cuts (Sec. 4.2): strips
    g = S.pd_structure(32, 32, [8], S.AXIS_X)
    assert len(g.leaves()) == 4 and all(r[0:2] == (0, 32) for r in g.rects)


def test_pd_errors():
    with pytest.raises(ValueError):
        S.pd_structure(8, 8, [8])         # no cut
    with pytest.raises(ValueError):
        S.pd_structure(8, 8, [])


def test_replica_colouring_on_overlapping_leaves():
    g = S.RegionGraph(num_vars=4)
    g.add_region(range(4))
    a = g.add_region((0, 1)); b = g.add_region((2, 3))
    c = g.add_region((0, 2)); d = g.add_region((1, 3))
    g.add_partition(0, a, b); g.add_partition(0, c, d)
    S.assign_replica_greedy(g)
    assert g.num_replica == 2 and g.replica == [-1, 0, 0, 1, 1]
    check_valid(g)


@pytest.mark.parametrize("g", [S.rat_structure(20, 3, 3, 5), S.pd_structure(28, 28, [7]),
                               S.pd_structure(64, 64, [16, 8]), S.pd_structure(6, 9, [3, 1])])
def test_topological_layers_properties(g):
    """What App. A states about the result of Algorithm 1."""
    sum_layers, prod_layers = S.topological_layers(g)
    assert len(sum_layers) == len(prod_layers)
    assert sum_layers[-1] == [0]                               # first iteration: only the root
    level_s = {s: i for i, layer in enumerate(sum_layers) for s in layer}
    level_p = {p: i for i, layer in enumerate(prod_layers) for p in layer}
    assert sorted(level_s) == [s for s in range(g.num_regions) if not g.is_leaf(s)]
    assert sorted(level_p) == list(range(g.num_partitions))
    for p, (parent, left, right) in enumerate(g.partitions):
        # the product layer holds exactly the children of the sum layer built in the same iteration
        assert level_p[p] == level_s[parent]
        for c in (left, right):
            if not g.is_leaf(c):
                assert level_s[c] < level_p[p]                 # inputs come from strictly lower layers
    # a sum is inserted as early (as high) as its parents allow: directly below its lowest parent
    for s in level_s:
        if s != 0:
            par = [level_p[p] for p, (_, l, r) in enumerate(g.partitions) if s in (l, r)]
            assert level_s[s] == min(par) - 1


def test_layer_sizes_of_benchmark_structures():
    _, pl = S.topological_layers(S.pd_structure(32, 32, [8]))
    assert [len(l) for l in pl] == [24, 50, 60, 40, 20, 6]
    _, pl = S.topological_layers(S.rat_structure(784, 8, 10, 1))
    assert [len(l) for l in pl] == [1280, 640, 320, 160, 80, 40, 20, 10]
