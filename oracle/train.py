"""Float64 oracle for what sits around one EM step: the stochastic-EM loop over
mini-batches (Eq. 8-9 with the schedule of Sec. 4.2) and the mixture of several
EiNets used for the image experiments (Sec. 4.2).

TEST INFRASTRUCTURE ONLY (see the package docstring).  Plain Python loops over
the definitions; pinned by tests/test_oracle_train.py: the one-entry Gaussian
or Bernoulli circuit reduces the loop to an exponential moving average of
mini-batch moments, and a mixture of normalised circuits is normalised.
"""
import numpy as np


def em_epoch(model, x, mask=None, batch=100, step=0.5, min_var=0.0, max_var=np.inf, w_floor=0.0):
    """One pass over the N samples of x in consecutive mini-batches (the last one
    may be shorter): for every mini-batch the statistics of Eq. 6 are taken under
    the current parameters and the parameters move by Eq. 8-9 with step size
    `step`, followed by the variance projection of Sec. 4.2.

    mask: None, [D] (shared by all samples) or [N, D] (one row per sample).
    Returns logP of every sample under the parameters in force when its
    mini-batch was visited (float64 [N]).  Updates `model` in place."""
    x = np.asarray(x, dtype=np.float64)
    N = x.shape[0]
    logp = np.empty(N)
    for b0 in range(0, N, batch):
        b1 = min(b0 + batch, N)
        mb = mask[b0:b1] if mask is not None and np.ndim(mask) == 2 else mask
        stats, lp = model.em_accumulate(x[b0:b1], mb)
        model.em_update(stats, step=step, min_var=min_var, max_var=max_var, w_floor=w_floor)
        logp[b0:b1] = lp
    return logp


def mixture_logp(component_logp, log_coef):
    """log sum_c coef_c * p_c(x_b) for component_logp [C][B] and log_coef [C] (Sec. 4.2:
    the components are EiNets, the coefficients the cluster proportions).  Written out
    with the usual shift by the largest term; a sample for which every term is -inf
    gets -inf."""
    t = np.asarray(component_logp, dtype=np.float64) + np.asarray(log_coef, dtype=np.float64)[:, None]
    C, B = t.shape
    out = np.empty(B)
    for b in range(B):
        m = -np.inf
        for c in range(C):
            m = max(m, t[c, b])
        if m == -np.inf:
            out[b] = -np.inf
            continue
        s = 0.0
        for c in range(C):
            s += np.exp(t[c, b] - m)
        out[b] = m + np.log(s)
    return out
