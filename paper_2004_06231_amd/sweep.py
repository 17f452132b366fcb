"""The efficiency sweeps of Sec. 4.1 (Fig. 3, and the inference-time figure of App. C) on one MI355X.

Random binary trees over D = 512 variables of synthetic Gaussian noise, N = 2000 samples, one-dimensional
Gaussian leaves; K, the split depth and the number of replica are varied one at a time around depth 4, R 10,
K 10.  For every point one JSON line: parameter count, training time per epoch (20 mini-batches of 100 samples,
one stochastic-EM update per mini-batch, Eq. 8-9), inference time per sample on a batch of 100 (batch time /
100, as in the paper) and the device memory the model holds (parameters + statistics + workspace; the data are
not counted).  The paper's own numbers are plots measured on another GPU; nothing is compared here.

    python -m paper_2004_06231_amd.sweep [--quick]
"""
import argparse
import json
import time

import numpy as np
import torch

import paper_2004_06231_amd as P
import workloads

N_TRAIN, BATCH = 2000, 100


def run_point(point, epochs=3):
    cfg = workloads.fig3_config(**point, B=BATCH)
    seed = 512
    m = P.EiNet(cfg["structure"], cfg["K"], 1, cfg["family"], BATCH, seed).bind("cuda:0")
    rng = np.random.default_rng(seed)
    m.init_params(seed, *cfg["leaf_range"])
    data = torch.as_tensor(workloads.draw_data(rng, cfg["data"], N_TRAIN, 512, 1)).cuda()
    batches = [data[i:i + BATCH].contiguous() for i in range(0, N_TRAIN, BATCH)]
    logp = torch.empty(BATCH, dtype=torch.float32, device="cuda")

    def epoch():
        for xb in batches:
            m.em_accumulate(xb, None, logp)
            m.em_update(step=0.5, min_var=1e-6, max_var=10.0, w_floor=1e-9)

    epoch()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(epochs):
        epoch()
    torch.cuda.synchronize()
    t_epoch = (time.perf_counter() - t0) / epochs
    for _ in range(5):
        m.logp(batches[0], None, logp)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(50):
        m.logp(batches[0], None, logp)
    torch.cuda.synchronize()
    t_inf = (time.perf_counter() - t0) / 50 / BATCH
    assert bool(torch.isfinite(logp).all())
    out = dict(point, n_params=m.n_params, train_s_per_epoch=round(t_epoch, 6),
               train_samples_per_s=round(N_TRAIN / t_epoch, 1), infer_us_per_sample=round(1e6 * t_inf, 3),
               model_mib=round((4 * (m.n_params + m.n_stats) + m.workspace_bytes) / 2 ** 20, 2))
    m.close()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--quick", action="store_true", help="only the ends and the centre of each sweep")
    args = ap.parse_args()
    ks = [1, 10, 40] if args.quick else [1, 2, 5, 10, 15, 20, 30, 40]
    ds = [1, 4, 9] if args.quick else list(range(1, 10))
    rs = [1, 10, 40] if args.quick else [1, 2, 5, 10, 20, 30, 40]
    for name, key, values in (("K", "K", ks), ("depth", "depth", ds), ("R", "R", rs)):
        for v in values:
            res = run_point({key: v})
            print(json.dumps(dict(sweep=name, **res)), flush=True)


if __name__ == "__main__":
    main()
