"""Float64 oracle for top-down sampling from an EiNet: ancestral sampling and sampling from
the conditional given evidence (inpainting), with leaf samples or leaf means (Sec. 2, the
latent-variable reading of smooth and decomposable circuits; Sec. 4.2; App. D).

TEST INFRASTRUCTURE ONLY (see the package docstring).  One sample at a time, plain loops.
Every random number is an input: one uniform per (partition, sample) and per (region,
sample) for the choices at the sums, one number per (sample, variable, channel) for the
leaves.  Pinned by tests/test_oracle_sampling.py (hand-computed choices, empirical
frequencies against the exact distribution and against Eq. 1, K = 1 closed forms).

The procedure.  A forward pass with the evidence (unobserved variables integrated out)
gives the value of every node.  Starting from the single entry of the root, a region with
entry k chooses one of its partitions n with probability v[k,n] * S_n[k] / N[k] (a region
with one partition has no choice), the partition chooses a pair (i, j) of entries of its
children with probability W[k,i,j] * N_left[i] * N_right[j] / S_n[k], and the two children
continue with i and j.  A leaf reached with entry k keeps its observed variables and fills
the others from its k-th distribution.  Without evidence all node values are 1 and the
choices follow the weights alone (ancestral sampling).

Choosing from unnormalised weights w_0..w_{n-1} with a uniform u: the first index t whose
running sum w_0 + ... + w_t exceeds u * (w_0 + ... + w_{n-1}); pairs (i, j) are numbered
i * K + j.  `margin` reports how close u came to a boundary of its interval, relative to the
total, so that a float32 implementation can be compared where the choice is not a toss-up.
"""
import numpy as np

from .einet import BERNOULLI, GAUSSIAN, BINOMIAL, CATEGORICAL, ef_log_density


def choose(w, u, other_side=False):
    """(index, margin) of the inverse-CDF choice described in the module docstring.  other_side: instead of the
    index whose interval holds u * total, its neighbour across the nearer boundary of that interval (the next
    index with a non-zero weight on that side, if there is one): what an implementation in lower precision may
    pick when the margin is tiny."""
    w = np.asarray(w, dtype=np.float64)
    c = np.cumsum(w)
    total = c[-1]
    tau = u * total
    t = int(np.searchsorted(c, tau, side="right"))        # first t with c[t] > tau
    if t >= len(w):                                       # u so close to 1 that rounding ate the last interval
        t = int(np.nonzero(w)[0][-1])
    lo = c[t - 1] if t > 0 else 0.0
    margin = min(tau - lo, c[t] - tau) / total
    if other_side:
        nz = np.nonzero(w)[0]
        side = nz[nz < t] if tau - lo <= c[t] - tau else nz[nz > t]
        if len(side):
            t = int(side[-1] if tau - lo <= c[t] - tau else side[0])
    return t, margin


def sample(model, B, u, noise=None, x=None, mask=None, only=None, flip=None, tie_margin=0.0):
    """Draws B samples.

    u     : [num_partitions + num_regions, B] uniforms in [0, 1): row n decides the pair of
            partition n, row num_partitions + s the partition of region s
    noise : [B, D, C]; Gaussian leaves: standard normal numbers, x = mean + sd * noise;
            Bernoulli leaves: uniforms, x = 1 if noise < p else 0; binomial and categorical
            leaves: uniforms, x = the first value whose running probability sum exceeds
            noise * (sum of all probabilities); None: the leaf means (E[x] of the chosen
            leaf entry, App. D)
    x, mask : evidence [B, D, C] and mask ([D] or [B, D], 1 = observed); None: no evidence

    only  : the samples to draw (default all; the others keep x, margin inf and an empty path)
    flip, tie_margin : flip = {b: j} takes, for sample b, the j-th (from 0, in the order the choices are made)
            of its choices whose margin is below tie_margin on the other side of the nearer boundary
            (`choose(..., other_side=True)`); the descent then continues from there.  For comparing
            implementations that decide near-ties in another precision.

    Returns (samples [B, D, C] float64 with the observed entries copied from x,
             margin [B]: the smallest margin over the choices made for each sample,
             paths: per sample the list of (partition, i, j) chosen).
    The evidence must have non-zero density."""
    g, K, C = model.g, model.K, model.C
    D, P = g.num_vars, g.num_partitions
    u = np.asarray(u, dtype=np.float64)
    assert u.shape == (P + g.num_regions, B)
    if x is None:
        x = np.zeros((B, D, C))
        mask = np.zeros(D)
    x = np.asarray(x, dtype=np.float64)
    m = model._mask(mask, B, D)
    _, N, S = model.forward(x, m)
    out = x.copy()
    margins = np.full(B, np.inf)
    paths = []
    for b in range(B):
        path = []
        if only is not None and b not in only:
            paths.append(path)
            continue
        ties = 0                                          # near-tie choices met so far
        want = None if flip is None else flip.get(b)

        def decide(w, ub):
            nonlocal ties
            t, mg = choose(w, ub)
            if mg < tie_margin:
                if want is not None and ties == want:
                    t, _ = choose(w, ub, other_side=True)
                ties += 1
            return t, mg

        todo = [(0, 0)]
        while todo:
            s, k = todo.pop()
            if g.is_leaf(s):
                r = g.replica[s]
                for d in g.scopes[s]:
                    if m[b, d]:
                        continue
                    for c in range(C):
                        phi = model.phi[d, c, r, :, k]
                        if noise is None:
                            if model.family == CATEGORICAL:
                                out[b, d, c] = float(np.dot(np.arange(model.leaf_param), phi))   # E[x]
                            else:
                                out[b, d, c] = phi[0]
                        elif model.family == GAUSSIAN:
                            out[b, d, c] = phi[0] + np.sqrt(phi[1] - phi[0] ** 2) * noise[b, d, c]
                        elif model.family == BERNOULLI:
                            out[b, d, c] = 1.0 if noise[b, d, c] < phi[0] else 0.0
                        else:
                            # discrete leaves: the first value whose cumulative probability exceeds the uniform
                            n_val = model.leaf_param + 1 if model.family == BINOMIAL else model.leaf_param
                            vals = np.arange(n_val, dtype=np.float64)
                            pmf = np.exp(ef_log_density(model.family, vals, phi[:, None], model.leaf_param))
                            out[b, d, c] = float(choose(pmf, noise[b, d, c])[0])
                continue
            parts = g.children[s]
            if len(parts) == 1:
                n = parts[0]
            else:
                w = np.array([model.v[s][k, ci] * np.exp(S[nn][b, k] - N[s][b, k]) for ci, nn in enumerate(parts)])
                ci, mg = decide(w, u[P + s, b])
                margins[b] = min(margins[b], mg)
                n = parts[ci]
            _, left, right = g.partitions[n]
            w = model.W[n][k] * np.exp(N[left][b][:, None] + N[right][b][None, :] - S[n][b, k])
            t, mg = decide(w.ravel(), u[n, b])
            margins[b] = min(margins[b], mg)
            i, j = divmod(t, K)
            path.append((n, i, j))
            todo.append((left, i))
            todo.append((right, j))
        paths.append(path)
    return out, margins, paths
