"""Stochastic-EM training of a mixture of EiNets as in the image experiments of Sec. 4.2, on one MI355X.

Every mixture component is an EiNet of its own, trained on its own share of the data (the paper clusters the
images with k-means; here every component gets a seeded synthetic cluster) for a number of epochs of
mini-batch EM (Eq. 8-9: batch 500, step 0.5, variances kept in [1e-6, 1e-2]); the mixture coefficients are the
cluster proportions.  The components are independent, so their epochs are enqueued round-robin on several HIP
streams of equal priority: one small circuit does not fill the chip, several side by side do.  With --graphs
every component's epoch (the same launches on the same buffers every time) is captured into a HIP graph after
the first epoch and replayed from then on, which takes the host's launch calls out of the loop.  Prints one
JSON line: training throughput over all epochs and over the epochs after the first (which also loads the
kernels), seconds per epoch, mean training logP of each epoch (first component) and the mean mixture logP of
a held-out batch.

    python -m paper_2004_06231_amd.train --shape svhn --components 8 --epochs 3 --n 5000 --streams 4 --graphs
"""
import argparse
import json
import time

import numpy as np
import torch

import paper_2004_06231_amd as P
import workloads


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--shape", default="svhn", choices=["svhn", "celeba"])
    ap.add_argument("--components", type=int, default=8)
    ap.add_argument("--epochs", type=int, default=3)
    ap.add_argument("--n", type=int, default=5000, help="training samples per component")
    ap.add_argument("--streams", type=int, default=4)
    ap.add_argument("--seed", type=int, default=42)
    ap.add_argument("--graphs", action="store_true", help="replay a captured HIP graph per component after the first epoch")
    args = ap.parse_args()
    cfg = workloads.sec42_config(args.shape)
    K, C, fam, B = cfg["K"], cfg["channels"], cfg["family"], cfg["B"]
    models, data, lps = [], [], []
    rng = np.random.default_rng(args.seed)
    sizes = rng.multinomial(args.n * args.components, rng.dirichlet(20.0 * np.ones(args.components)))
    sizes = np.maximum(sizes, B)
    for c in range(args.components):
        m = P.EiNet(cfg["structure"], K, C, fam, B, args.seed + c).bind("cuda:0")
        D = int(m.structure()["num_vars"])
        m.init_params(args.seed + c, *cfg["leaf_range"])
        data.append(torch.as_tensor(workloads.draw_data(rng, cfg["data"], int(sizes[c]), D, C)).cuda())
        lps.append(torch.empty(int(sizes[c]), dtype=torch.float32, device="cuda"))
        models.append(m)
    held_out = torch.cat([d[:B // args.components + 1] for d in data])[:B].contiguous()
    streams = [torch.cuda.Stream() for _ in range(max(1, args.streams))]
    torch.cuda.synchronize()

    def epoch():
        for c, m in enumerate(models):
            with torch.cuda.stream(streams[c % len(streams)]):
                m.em_epoch(data[c], None, batch=B, logp=lps[c], **cfg["em"])

    graphs = []

    def capture():
        # A component's epoch as a graph: between replays nothing else may touch the component (its statistics
        # are empty and its root posterior in place at the start of every epoch, as they were at capture).
        for c, m in enumerate(models):
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=streams[c % len(streams)]):
                m.em_epoch(data[c], None, batch=B, logp=lps[c], **cfg["em"])
            graphs.append(g)
        torch.cuda.synchronize()

    def replay():
        for c, g in enumerate(graphs):
            with torch.cuda.stream(streams[c % len(streams)]):
                g.replay()

    history, seconds = [], []
    t0 = time.perf_counter()
    for e in range(args.epochs):
        t1 = time.perf_counter()
        if graphs:
            replay()
        else:
            epoch()
        torch.cuda.synchronize()
        seconds.append(round(time.perf_counter() - t1, 4))
        history.append(round(float(lps[0].mean()), 3))
        if args.graphs and e == 0 and args.epochs > 1:
            capture()                                    # (its time counts in the total, not in an epoch's)
    dt = time.perf_counter() - t0
    # mixture of the trained components on a held-out batch
    rows = torch.empty(args.components, held_out.shape[0], dtype=torch.float32, device="cuda")
    for c, m in enumerate(models):
        m.logp(held_out, None, rows[c])
    log_coef = torch.as_tensor(np.log(sizes / sizes.sum()), dtype=torch.float32).cuda()
    mix = P.einet_mixture_logp(rows, log_coef)
    assert bool(torch.isfinite(mix).all()) and all(bool(torch.isfinite(m.params).all()) for m in models)
    total = int(sizes.sum()) * args.epochs
    later = sum(seconds[1:])
    print(json.dumps(dict(workload=cfg["name"], components=args.components, streams=len(streams), epochs=args.epochs,
                          graphs=bool(graphs),
                          samples_per_component=[int(s) for s in sizes], n_params_per_component=models[0].n_params,
                          train_samples_per_s=round(total / dt, 1), seconds=round(dt, 4), seconds_per_epoch=seconds,
                          samples_per_s_after_first_epoch=round(int(sizes.sum()) * (args.epochs - 1) / later, 1) if later > 0 else None,
                          train_mean_logp_per_epoch_component0=history,
                          held_out_mixture_mean_logp=round(float(mix.mean()), 3))))
    for m in models:
        m.close()


if __name__ == "__main__":
    main()
