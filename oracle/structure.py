"""Region graphs for the oracle (test infrastructure, float64 CPU side only).

A vectorised probabilistic circuit (Sec. 3.1) is held as a *region graph*:

* a region is a set of variables (its scope); it stands for a vector of K
  densities over that scope: a leaf if it has no partitions, otherwise a sum
  node whose children are its partitions;
* a partition is a product node with exactly two child regions (left, right)
  of disjoint scope whose union is the scope of the one region it belongs to
  (each product has a single parent, Sec. 3.1).

The two generators are the structures the paper experiments with: random
binary trees (Sec. 4.1) and the Poon-Domingos image structure (Sec. 4.2).
Where the paper leaves the construction open, the numbering and the random
number generator below are this build's own convention; the C library follows
the same written convention in code of its own, and the tests compare the two
structures integer by integer.

Conventions
-----------
Random binary trees, ``rat_structure(D, depth, R, seed)``:
  region 0 is the root (scope 0..D-1).  Replica r is a complete binary tree;
  its node with heap index h (root h=1, children 2h and 2h+1) is, for h >= 2,
  region ``1 + r*(2**(depth+1)-2) + (h-2)``.  The split of heap node h
  (1 <= h < 2**depth) of replica r is partition ``r*(2**depth-1) + (h-1)``.
  A scope of n variables, sorted ascending, is shuffled with Fisher-Yates
  (t = n-1 .. 1: swap a[t], a[u mod (t+1)]) driven by a SplitMix64 stream
  whose initial state is ``seed ^ (C1*(r+1)) ^ (C2*h)`` (64-bit wrap); the
  first n//2 shuffled variables (sorted) go left, the rest (sorted) right.
Poon-Domingos, ``pd_structure(H, W, deltas, axes)``:
  variable index of pixel (y, x) is y*W + x.  Regions are rectangles
  [y0,y1) x [x0,x1); region 0 is the image.  Rectangles are processed in
  creation (breadth-first) order.  For a rectangle the step is the first
  delta in ``deltas`` that gives at least one cut on an allowed axis; cuts
  are taken first along y (y0+m*delta, ascending), then along x, and each cut
  is a partition (top|left rectangle = left child).  Child rectangles get
  the next free region number the first time they are seen (left before
  right); partitions are numbered in creation order.
"""
from __future__ import annotations

from dataclasses import dataclass, field

MASK64 = (1 << 64) - 1
_C1 = 0xD1B54A32D192ED03
_C2 = 0x8CB92BA72F3D8DD7

AXIS_Y = 1  # cuts that separate rows   (a horizontal line)
AXIS_X = 2  # cuts that separate columns (a vertical line)


class SplitMix64:
    """SplitMix64 (Steele, Lea, Flood 2014; Vigna's public-domain constants)."""

    def __init__(self, state: int):
        self.state = state & MASK64

    def next(self) -> int:
        self.state = (self.state + 0x9E3779B97F4A7C15) & MASK64
        z = self.state
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & MASK64
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & MASK64
        return z ^ (z >> 31)


@dataclass
class RegionGraph:
    num_vars: int
    scopes: list = field(default_factory=list)        # region -> sorted tuple of variables
    partitions: list = field(default_factory=list)    # partition -> (parent, left, right)
    children: list = field(default_factory=list)      # region -> list of its partitions
    replica: list = field(default_factory=list)       # region -> replica (leaf) or -1
    num_replica: int = 0
    rects: list | None = None                         # PD only: region -> (y0, y1, x0, x1)

    @property
    def num_regions(self):
        return len(self.scopes)

    @property
    def num_partitions(self):
        return len(self.partitions)

    def is_leaf(self, s):
        return len(self.children[s]) == 0

    def leaves(self):
        return [s for s in range(self.num_regions) if self.is_leaf(s)]

    def k_out(self, s, K):
        """Vector length of region s: 1 at the root, K elsewhere (root is a
        single density, Sec. 2; fixed by the parameter counts of Fig. 3)."""
        return 1 if s == 0 else K

    def add_region(self, scope):
        self.scopes.append(tuple(scope))
        self.children.append([])
        self.replica.append(-1)
        return len(self.scopes) - 1

    def add_partition(self, parent, left, right):
        self.partitions.append((parent, left, right))
        self.children[parent].append(len(self.partitions) - 1)
        return len(self.partitions) - 1


def rat_split(scope, seed, r, h):
    """Random balanced split of a sorted scope (Sec. 4.1)."""
    a = list(scope)
    n = len(a)
    rng = SplitMix64((seed ^ ((_C1 * (r + 1)) & MASK64) ^ ((_C2 * h) & MASK64)) & MASK64)
    for t in range(n - 1, 0, -1):
        j = rng.next() % (t + 1)
        a[t], a[j] = a[j], a[t]
    return tuple(sorted(a[: n // 2])), tuple(sorted(a[n // 2:]))


def rat_structure(D, depth, R, seed):
    """R random binary trees of the given split depth, mixed at the root (Sec. 4.1)."""
    if D < 2 or depth < 1 or R < 1:
        raise ValueError("need D >= 2, depth >= 1, R >= 1")
    g = RegionGraph(num_vars=D)
    g.add_region(range(D))
    per_tree = 2 ** (depth + 1) - 2
    # reserve regions so the closed-form numbering holds whatever order we fill them in
    for _ in range(R * per_tree):
        g.add_region(())
    parts = [None] * (R * (2 ** depth - 1))
    for r in range(R):
        def rid(h):
            return 0 if h == 1 else 1 + r * per_tree + (h - 2)
        for h in range(1, 2 ** depth):
            scope = g.scopes[rid(h)]
            if len(scope) < 2:
                raise ValueError("depth too large: a scope of one variable cannot be split")
            left, right = rat_split(scope, seed, r, h)
            g.scopes[rid(2 * h)] = left
            g.scopes[rid(2 * h + 1)] = right
            parts[r * (2 ** depth - 1) + (h - 1)] = (rid(h), rid(2 * h), rid(2 * h + 1))
        for h in range(2 ** depth, 2 ** (depth + 1)):
            g.replica[rid(h)] = r
    for p in parts:
        g.add_partition(*p)
    g.num_replica = R
    return g


def _pd_cuts(rect, deltas, axes):
    y0, y1, x0, x1 = rect
    for d in deltas:
        ys = list(range(y0 + d, y1, d)) if axes & AXIS_Y else []
        xs = list(range(x0 + d, x1, d)) if axes & AXIS_X else []
        if ys or xs:
            return ys, xs
    return [], []


def pd_structure(H, W, deltas, axes=AXIS_Y | AXIS_X):
    """Poon-Domingos structure: recursive axis-aligned cuts displaced by a step (Sec. 4.2)."""
    deltas = list(deltas)
    if H < 1 or W < 1 or not deltas or min(deltas) < 1 or not (axes & 3):
        raise ValueError("bad PD arguments")
    g = RegionGraph(num_vars=H * W, rects=[])

    def scope_of(rect):
        y0, y1, x0, x1 = rect
        return tuple(y * W + x for y in range(y0, y1) for x in range(x0, x1))

    ids = {}

    def get(rect):
        if rect not in ids:
            ids[rect] = g.add_region(scope_of(rect))
            g.rects.append(rect)
        return ids[rect]

    get((0, H, 0, W))
    s = 0
    while s < g.num_regions:
        rect = g.rects[s]
        y0, y1, x0, x1 = rect
        ys, xs = _pd_cuts(rect, deltas, axes)
        for c in ys:
            left = get((y0, c, x0, x1))
            right = get((c, y1, x0, x1))
            g.add_partition(s, left, right)
        for c in xs:
            left = get((y0, y1, x0, c))
            right = get((y0, y1, c, x1))
            g.add_partition(s, left, right)
        s += 1
    if g.is_leaf(0):
        raise ValueError("no step in deltas cuts the image")
    assign_replica_greedy(g)
    return g


def assign_replica_greedy(g):
    """Give each leaf region the smallest replica index not used by an
    overlapping leaf that was numbered earlier, so that leaves sharing a
    replica have disjoint scopes (Sec. 3.4)."""
    used = []  # replica -> set of variables already covered
    for s in g.leaves():
        sc = set(g.scopes[s])
        for r, cov in enumerate(used):
            if not (cov & sc):
                cov |= sc
                g.replica[s] = r
                break
        else:
            used.append(set(sc))
            g.replica[s] = len(used) - 1
    g.num_replica = len(used)


def topological_layers(g):
    """Algorithm 1 (App. A): top-down breadth-first layering.

    Returns (sum_layers, product_layers), each a list of sorted lists, ordered
    bottom-up (index 0 is the lowest internal layer).  Sum nodes are the
    non-leaf regions, product nodes are the partitions.  A region's parents
    are the partitions it is a child of; a partition's parent is its region.
    """
    sums = {s for s in range(g.num_regions) if not g.is_leaf(s)}
    prods = set(range(g.num_partitions))
    parents_of_sum = {s: set() for s in sums}
    for p, (_, left, right) in enumerate(g.partitions):
        for c in (left, right):
            if c in parents_of_sum:
                parents_of_sum[c].add(p)
    visited_s, visited_p = set(), set()
    sum_layers, prod_layers = [], []
    while visited_s != sums or visited_p != prods:
        ls = {s for s in sums if s not in visited_s and parents_of_sum[s] <= visited_p}
        sum_layers.insert(0, sorted(ls))
        visited_s |= ls
        lp = {p for p in prods if p not in visited_p and g.partitions[p][0] in visited_s}
        prod_layers.insert(0, sorted(lp))
        visited_p |= lp
        if not ls and not lp:
            raise ValueError("graph is not a rooted DAG of alternating sums and products")
    return sum_layers, prod_layers


@dataclass
class ParamLayout:
    """Offsets (in floats) into the flat parameter and statistics buffers.

    parameters: [ W | v | phi ]
      W   : partitions in order, each [K_out][K][K] (j fastest)
      v   : regions with more than one partition, in order, each [K_out][C_s]
      phi : [D][C][R][T][K] expectation parameters (T=1 Bernoulli, 2 Gaussian)
    statistics: [ Nw | Nv | num | den | tot ]
      Nw, Nv, num : same shapes as W, v, phi
      den, tot    : [D][R][K]
    """
    w_off: list
    v_off: dict
    phi_off: int
    n_params: int
    den_off: int
    tot_off: int
    n_stats: int


def param_layout(g, K, C, T):
    off = 0
    w_off = []
    for (parent, _, _) in g.partitions:
        w_off.append(off)
        off += g.k_out(parent, K) * K * K
    v_off = {}
    for s in range(g.num_regions):
        if len(g.children[s]) > 1:
            v_off[s] = off
            off += g.k_out(s, K) * len(g.children[s])
    phi_off = off
    off += g.num_vars * C * g.num_replica * T * K
    n_params = off
    den_off = off
    tot_off = den_off + g.num_vars * g.num_replica * K
    n_stats = tot_off + g.num_vars * g.num_replica * K
    return ParamLayout(w_off, v_off, phi_off, n_params, den_off, tot_off, n_stats)
