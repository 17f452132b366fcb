#!/usr/bin/env python3
"""Benchmark of the EiNet hot path on one MI355X.

A step is one full EM step on one resident batch of synthetic data: forward pass
(leaf, einsum and mixing layers), top-down pass accumulating the expected
statistics, and the M-step.  The workload is configuration 4 (Poon-Domingos
structure on a 32x32x3 grid, step 8, K=40, Gaussian leaves, B=128), the largest of
the five configurations in einsum work; the data stand in for 32x32 RGB images and
are drawn from a seeded Gaussian mixture.

Prints ONE JSON line: EM samples/s as `value`, plus logP samples/s, the per-kernel
device times, the roofline of the dominant kernel, and the float64 oracle timed on
a bounded sample of the same batch on the host cores.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0          # MI355X HBM3E
PEAK_MFMA_FP32_TFLOPS = 157.3  # MI355X dense fp32 matrix rate
WORKLOAD = 4


def measured_traffic(workload, kernel):
    """HBM bytes per launch of a kernel class on a configuration, as the committed counter summary states it
    (profiles/hbm_traffic_cfg<N>.md, line `traffic_bytes_per_launch <kernel class> <bytes>`, written from two
    rocprofv3 --pmc runs); None when there is no such measurement."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_cfg{workload}.md")
    try:
        with open(path) as f:
            for line in f:
                w = line.split()
                if len(w) >= 3 and w[0] == "traffic_bytes_per_launch" and w[1] == kernel:
                    return float(w[2])
    except OSError:
        pass
    return None


def algorithmic_work(st, K, C, R, T, TD, B, D):
    """Per step, per kernel class: (flop, bytes) the method itself needs (unpadded K, no
    materialised outer products, every operand moved once)."""
    part = st["partition"]
    kout = [1 if p[0] == 0 else K for p in part]
    n_children = {}
    for p in part:
        n_children[p[0]] = n_children.get(p[0], 0) + 1
    mix = {s: c for s, c in n_children.items() if c > 1}
    n_leaf = int((st["region_replica"] >= 0).sum())
    w = {}
    # the root's partitions (one output entry each) and the root's mixture run in launches of their own
    inner = [ko for ko in kout if ko != 1] if K != 1 else kout
    top = [ko for ko in kout if ko == 1] if K != 1 else []
    w["einsum_forward"] = (sum(2.0 * B * ko * K * K for ko in inner),
                           sum(4.0 * ko * K * K + 4.0 * B * (2 * K + ko) for ko in inner))
    # backward: W read, Nw written (after an M-step the statistics start from zero, so the benchmark loop
    # never has to read them back); L, R, A_out, G_out read; two posterior blocks written
    w["einsum_backward"] = (sum(4.0 * B * ko * K * K for ko in inner),
                            sum(8.0 * ko * K * K + 4.0 * B * (4 * K + 2 * ko) for ko in inner))
    w["root_forward"] = (sum(2.0 * B * K * K for _ in top),
                         sum(4.0 * K * K + 4.0 * B * (2 * K + 1) for _ in top) + 4.0 * B)
    w["root_backward"] = (sum(4.0 * B * K * K for _ in top),
                          sum(8.0 * K * K + 4.0 * B * (4 * K + 2) for _ in top))
    w["mixing_forward"] = (0.0, sum(4.0 * (c + 1) * B * K for s, c in mix.items() if s != 0))
    w["leaf_forward"] = (0.0, 4.0 * B * D * C + 4.0 * D * C * R * TD * K + 4.0 * n_leaf * B * K)
    w["leaf_mixing_backward"] = (0.0, 4.0 * B * D * C + 4.0 * n_leaf * B * K + 8.0 * (D * C * R * T * K + 2 * D * R * K)
                                 + sum(4.0 * (c + 2) * B * (1 if s == 0 else K) for s, c in mix.items()))
    n_param = float(st["phi_offset"]) + D * C * R * T * K
    w["em_update"] = (0.0, 4.0 * 3 * n_param)       # read statistics and parameters, write parameters (+ zeroing)
    n_regions = st["num_regions"]
    w["region_backward"] = (0.0, 4.0 * B * K * (n_regions + 2 * len(part)))
    return w


def profiled_pass(m, em_step, steps, work):
    """Runs `steps` EM steps with a HIP event pair around every launch (recorded on the stream the kernels run on;
    a separate pass, since recording costs host time).  Returns the per-class table, the roofline of the class with
    the largest device time, and the launches one by one."""
    import torch
    m.profile_enable(True)
    for _ in range(steps):
        em_step()
    torch.cuda.synchronize()
    prof = m.profile_read()
    launch_list = m.profile_launches()
    m.profile_enable(False)
    kernels = {}
    for name, (ms, launches) in prof.items():
        if launches == 0:
            continue
        flop, byts = work[name]
        per_step_us = 1e3 * ms / steps
        kernels[name] = dict(us_per_step=round(per_step_us, 2), launches_per_step=launches // steps,
                             tflops=round(flop / (per_step_us * 1e-6) / 1e12, 3),
                             gbs=round(byts / (per_step_us * 1e-6) / 1e9, 1))
    dom = max(kernels, key=lambda n: kernels[n]["us_per_step"])
    flop, byts = work[dom]
    n_launch = kernels[dom]["launches_per_step"]
    avg_launch_s = kernels[dom]["us_per_step"] * 1e-6 / n_launch
    # which roof binds the dominant kernel: the one that takes longer at peak
    if flop / (PEAK_MFMA_FP32_TFLOPS * 1e12) >= byts / (PEAK_HBM_GBS * 1e9):
        achieved = flop / n_launch / avg_launch_s / 1e12
        roof = dict(bound="mfma", achieved=round(achieved, 3), peak=PEAK_MFMA_FP32_TFLOPS, unit="TFLOP/s",
                    frac=round(achieved / PEAK_MFMA_FP32_TFLOPS, 4))
    else:
        achieved = byts / n_launch / avg_launch_s / 1e9
        roof = dict(bound="hbm", achieved=round(achieved, 1), peak=PEAK_HBM_GBS, unit="GB/s",
                    frac=round(achieved / PEAK_HBM_GBS, 4))
    roof.update(kernel=dom, avg_launch_us=round(avg_launch_s * 1e6, 2), launches_per_step=n_launch,
                algorithmic_flop_per_step=flop, algorithmic_bytes_per_step=byts,
                algorithmic_bytes_per_launch=round(byts / n_launch, 1))
    return kernels, roof, launch_list


def time_config(i, steps, warmup):
    """EM-step and logP rates of configuration i (1-based) with its own seeded inputs."""
    import numpy as np
    import torch
    import paper_2004_06231_amd as P
    import workloads
    cfg = workloads.get_config(i)
    seed = workloads.config_seed(i)
    K, C, fam, B = cfg["K"], cfg["channels"], cfg["family"], cfg["B"]
    m = P.EiNet(cfg["structure"], K, C, fam, B, seed).bind("cuda:0")
    st = m.structure()
    D, R, T = st["num_vars"], st["num_replica"], st["T"]
    rng = np.random.default_rng(seed)
    flat = workloads.draw_params(rng, m.n_params, m.weight_blocks(), int(st["phi_offset"]), (D, C, R, T, K), fam,
                                 cfg["leaf_range"])
    x = torch.as_tensor(workloads.draw_data(rng, cfg["data"], B, D, C)).cuda()
    mask = workloads.draw_mask(rng, cfg["mask"], B, D)
    mask = None if mask is None else torch.as_tensor(mask).cuda()
    m.set_params(flat)
    logp = torch.empty(B, dtype=torch.float32, device="cuda")
    kw = dict(step=0.5, min_var=1e-6, max_var=1e-2, w_floor=1e-9) if fam == P.GAUSSIAN else dict(step=0.5, w_floor=1e-9)
    res = {"batch": B, "n_params": m.n_params}
    for name, fn in (("em", lambda: (m.em_accumulate(x, None, logp), m.em_update(**kw))),
                     ("logp", lambda: m.logp(x, mask, logp))):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / steps
        res[name + "_samples_per_s"] = round(B / dt, 1)
        res[name + "_ms"] = round(1e3 * dt, 4)
    TD = 3 if fam == P.GAUSSIAN else 2
    work = algorithmic_work(st, K, C, R, T, TD, B, D)
    kernels, roof, _ = profiled_pass(m, lambda: (m.em_accumulate(x, None, logp), m.em_update(**kw)), steps, work)
    res["roofline"] = {k: roof[k] for k in ("kernel", "bound", "achieved", "peak", "unit", "frac", "avg_launch_us",
                                            "launches_per_step")}
    res["kernels_us_per_step"] = {k: v["us_per_step"] for k, v in kernels.items()}
    m.close()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-configs", action="store_true")
    ap.add_argument("--no-peaks", action="store_true", help="skip the streaming-copy and register-resident MFMA loops")
    ap.add_argument("--workload", type=int, default=WORKLOAD, help="configuration to time (1-5); the default is the headline")
    ap.add_argument("--batch", type=int, default=0,
                    help="batch size instead of the configuration's own (for batch-scaling tables; not the headline)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only; sharding over the batch with one all-reduce of the "
              "statistics per M-step is how it would scale out; that is not built. Use --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2004_06231_amd as P
    import workloads

    wl = args.workload
    cfg = workloads.get_config(wl)
    seed = workloads.config_seed(wl)
    K, C, fam, B = cfg["K"], cfg["channels"], cfg["family"], args.batch or cfg["B"]
    m = P.EiNet(cfg["structure"], K, C, fam, B, seed).bind("cuda:0")
    st = m.structure()
    D, R, T = st["num_vars"], st["num_replica"], st["T"]
    TD = 3 if fam == P.GAUSSIAN else 2
    rng = np.random.default_rng(seed)
    flat = workloads.draw_params(rng, m.n_params, m.weight_blocks(), int(st["phi_offset"]), (D, C, R, T, K), fam,
                                 cfg["leaf_range"])
    x_host = workloads.draw_data(rng, cfg["data"], B, D, C)
    m.set_params(flat)
    x = torch.as_tensor(x_host).cuda()
    logp = torch.empty(B, dtype=torch.float32, device="cuda")
    em_kw = dict(step=0.5, min_var=1e-6, max_var=1e-2, w_floor=1e-9)   # Sec. 4.2 settings

    def em_step():
        m.em_accumulate(x, None, logp)
        m.em_update(**em_kw)

    # one device-to-device copy of the parameter buffer: a kernel of known size (n_params*4 bytes read and
    # written) against which the HBM byte counters of a rocprofv3 --pmc run are scaled
    calib = m.params.clone()
    del calib

    for _ in range(args.warmup):
        em_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        em_step()
    torch.cuda.synchronize()
    t_em = time.perf_counter() - t0
    ms_per_step = 1e3 * t_em / args.steps

    # forward only
    for _ in range(args.warmup):
        m.logp(x, None, logp)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        m.logp(x, None, logp)
    torch.cuda.synchronize()
    t_lp = time.perf_counter() - t0

    # top-down sampling (random numbers generated beforehand, not timed): without evidence, and inpainting of the
    # half of the variables that a shared mask hides, with leaf means
    n_choices = int(st["num_partitions"]) + int(st["num_regions"])
    u_rand = torch.rand(n_choices, B, device="cuda")
    noise = torch.randn(B, D, C, device="cuda") if fam == P.GAUSSIAN else torch.rand(B, D, C, device="cuda")
    half = torch.zeros(D, dtype=torch.uint8, device="cuda")
    half[: D // 2] = 1
    x_out = torch.empty_like(x)
    sampling = {}
    for name, fn in (("unconditional", lambda: m.sample(B, u_rand, noise, None, None, x_out)),
                     ("inpainting_means", lambda: m.sample(B, u_rand, None, x, half, x_out))):
        for _ in range(args.warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            fn()
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / args.steps
        sampling[name] = {"samples_per_s": round(B / dt, 1), "ms_per_call": round(1e3 * dt, 4)}
    assert bool(torch.isfinite(x_out).all())

    work = algorithmic_work(st, K, C, R, T, TD, B, D)
    kernels, roof, launch_list = profiled_pass(m, em_step, args.steps, work)
    dom = roof["kernel"]
    roof.update(traffic=measured_traffic(wl, dom) if B == cfg["B"] else None,
                traffic_unit="HBM bytes per launch (rocprofv3 counters, profiles/hbm_traffic_cfg%d.md)" % wl,
                timing="hip events around each launch, separate pass of the same steps")

    # launch by launch: the einsum layers of one step, averaged over the steps of the profiled pass (the work tag of
    # a launch is the number of output entries summed over its partitions)
    # (the root's partitions, one output entry each, have launches of their own: root_forward, which also forms the
    # root's mixture, and root_backward)
    ein = [l for l in launch_list if l[0] in ("einsum_forward", "einsum_backward", "root_forward", "root_backward")]
    per_step = len(ein) // args.steps
    layers = []
    if per_step * args.steps == len(ein):
        for pos in range(per_step):
            name, _, tag = ein[pos]
            outs, parts = tag >> 24, tag & 0xFFFFFF
            us = 1e3 * sum(ein[s_ * per_step + pos][1] for s_ in range(args.steps)) / args.steps
            fwd = name.endswith("_forward")
            fl = (2.0 if fwd else 4.0) * B * K * K * outs
            # W once (and Nw written once top-down); rows of the children, of the region and its posterior; outputs
            by = (4.0 if fwd else 8.0) * K * K * outs + 4.0 * B * ((2 * K * parts + outs) if fwd else (4 * K * parts + 2 * outs))
            layers.append(dict(kernel=name, outputs=int(outs), partitions=int(parts), us=round(us, 2),
                               tflops=round(fl / us / 1e6, 2), frac=round(fl / us / 1e6 / PEAK_MFMA_FP32_TFLOPS, 4),
                               gbs=round(by / us / 1e3, 1), frac_hbm=round(by / us / 1e3 / PEAK_HBM_GBS, 4)))
    roof["einsum_layers"] = layers

    if not args.no_peaks:
        pk = P.measure_peaks()
        roof["measured_peaks"] = {k: round(v, 1) for k, v in pk.items()}
        if roof["bound"] == "mfma":
            roof["frac_of_measured_peak"] = round(roof["achieved"] / pk["mfma_f32_32x32x2_tflops"], 4)
        else:
            roof["frac_of_measured_peak"] = round(roof["achieved"] / pk["copy_gbs"], 4)

    out = {
        "metric": "EM samples/sec (fwd+bwd+M-step)", "value": round(B * args.steps / t_em, 1), "unit": "samples/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": cfg["name"], "structure": cfg["structure"], "K": K, "batch": B,
                   "leaves": "gaussian" if fam == P.GAUSSIAN else "bernoulli", "em": em_kw},
        "logp_samples_per_s": round(B * args.steps / t_lp, 1), "logp_ms_per_call": round(1e3 * t_lp / args.steps, 4),
        "sampling": sampling,
        "kernels": kernels,
        "roofline": roof,
    }

    if not args.no_other_configs:
        # the other four configurations, for context (same protocol, fewer steps; not the headline value)
        out["other_configs"] = {}
        for i in [j for j in (1, 2, 3, 4, 5) if j != wl]:
            out["other_configs"][workloads.get_config(i)["name"]] = time_config(i, max(5, args.steps // 3), args.warmup)

    if not args.no_cpu_baseline:
        # the float64 oracle, as it stands, on a bounded sample of the same batch
        from tests.common import make_config
        _, oracle, _, xs, _ = make_config(wl, batch=B)
        assert np.array_equal(xs, x_host)
        t0 = time.perf_counter()
        stats, _ = oracle.em_accumulate(xs, None, chunk=8)
        oracle.em_update(stats, **em_kw)
        t_cpu = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(B / t_cpu, 3), "unit": "samples/s", "cores": 1, "kind": "oracle",
                               "sample": f"one EM step on the whole batch of {B} samples of {cfg['name']} "
                                         f"(float64 NumPy, single thread), {t_cpu:.1f} s"}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
