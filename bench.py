#!/usr/bin/env python3
"""Benchmark of one partition's sampled mini-batch step on one MI355X.

A step = the whole hot path over one batch of synthetic input: for every GCN layer, top-down,
csgs_build_probs -> csgs_sample_layer -> csgs_remote_count; then, bottom-up, csgs_aggregate ->
csgs_layer_gemm.  Inputs are resident in HBM before the timed region.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config large]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

HBM_PEAK_GBS = 8000.0
MFMA_F32_PEAK_TFLOPS = 157.3


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="large")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--scale", type=int, default=1, help="multiply batch and samples per layer (scaled-up variant)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (one partition's share); --gpus above 1 is not supported",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2101_07706_amd import csgs, pipeline, synth

    csgs.lib()  # fail loudly if the HIP library is missing
    assert torch.cuda.is_available(), "needs a GPU"
    dev = torch.device("cuda:0")
    cfg = synth.CONFIGS[args.config]
    if args.scale != 1:
        import dataclasses
        cfg = dataclasses.replace(cfg, batch=cfg.batch * args.scale, samples=cfg.samples * args.scale)
    bf16 = cfg.feat_dtype == "bf16"
    t0 = time.time()
    g = synth.make_graph(cfg)
    log(f"graph {cfg.name}: N={g.n_nodes} nnz={g.nnz} local=[{g.local_lo},{g.local_hi}) in {time.time() - t0:.1f}s")
    X = synth.make_features(cfg.n_nodes, cfg.feat_dim, cfg.seed)
    dims = synth.layer_dims(cfg)
    Ws = [synth.glorot_uniform(fi, fo, cfg.seed) for fi, fo in dims]
    M = len(dims)
    B = cfg.samples
    n_batches = args.steps + args.warmup
    batches = [synth.make_batch(g, cfg.batch, cfg.seed, it) for it in range(n_batches)]
    seed = 1234 + cfg.seed

    dg = pipeline.DeviceGraph(g, dev)
    Xh = synth.to_bf16_bits(X).view(np.int16) if bf16 else X
    Xd = torch.from_numpy(Xh).to(dev)
    X_local = Xd[g.local_lo:g.local_hi]
    Wd = [torch.from_numpy(W).to(dev) for W in Ws]
    Sd = [torch.from_numpy(b).to(dev) for b in batches]
    nS_max = max(cfg.batch, B)
    ws = pipeline.Workspace(g.n_nodes, nS_max, B, g.nnz, dev)
    adj_cap = int(min(g.nnz, 48_000_000))
    lbs = [pipeline.LayerBuffers(nS_max, B, g.n_nodes, adj_cap, dg.n_parts, dev) for _ in range(M)]
    Zs = [torch.empty((nS_max, dims[M - 1 - l][0]), dtype=torch.float32, device=dev) for l in range(M)]
    Hs = [torch.empty((nS_max, dims[M - 1 - l][1]), dtype=torch.float32, device=dev) for l in range(M)]
    counts_pinned = torch.zeros(2, dtype=torch.int64).pin_memory()
    elt = 2 if bf16 else 4
    log(f"inputs resident: {torch.cuda.memory_allocated() / 2**30:.2f} GiB")

    def step(it, sizes=None):
        """One whole mini-batch.  The host learns each layer's sampled-set size (it sizes the next launch)."""
        S = Sd[it]
        rows = []
        for l in range(M):
            lb = lbs[l]
            pipeline.sample_step(dg, ws, S, cfg.skew, B, seed, it, l, lb, want_q=False)
            n = int(lb.n_next.item())
            rows.append(S)
            S = lb.S_next[:n]
        r = int(lbs[M - 1].remote_total.item())
        X_remote = Xd[lbs[M - 1].remote_ids[:r].long()]      # stands in for the exchange of remote rows
        H = None
        for l in range(M - 1, -1, -1):
            lb = lbs[l]
            nS = rows[l].numel()
            Z, Hn = Zs[l][:nS], Hs[l][:nS]
            if l == M - 1:
                pipeline.compute_step(lb, nS, X_local, X_remote, True, False, Wd[M - 1 - l], Z, Hn)
            else:
                pipeline.compute_step(lb, nS, H, None, False, True, Wd[M - 1 - l], Z, Hn)
            H = Hn
        if sizes is not None:
            torch.cuda.synchronize()
            for l in range(M):
                st = lbs[l].stats_host()
                sizes.append(dict(layer=l, nS=rows[l].numel(), E=st.edges_scanned, nc=st.n_cand,
                                  n_next=int(lbs[l].n_next.item()), nnz=int(lbs[l].adj_nnz.item()),
                                  remote=int(lbs[l].remote_total.item()), F_in=dims[M - 1 - l][0],
                                  F_out=dims[M - 1 - l][1], elt=elt if l == M - 1 else 4,
                                  status=int(lbs[l].status.item())))
        return H

    for it in range(args.warmup):
        step(it)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for it in range(args.warmup, n_batches):
        step(it)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3
    log(f"timed {args.steps} steps: {ms_per_step:.3f} ms/step")

    # same steps again with every kernel launch bracketed by HIP events (on the launch stream)
    sizes = []
    csgs.csgs_profile_enable(True)
    for it in range(args.warmup, n_batches):
        step(it, sizes)
    torch.cuda.synchronize()
    csgs.csgs_profile_enable(False)
    prof = csgs.csgs_profile_collect()
    assert all(s["status"] == 0 for s in sizes), "a status bit was set"

    # algorithmic bytes / flops per kernel, summed over the launches of the profiled region
    N = g.n_nodes
    alg = {k: 0.0 for k in prof}
    flops = 0.0
    for s in sizes:
        nS, E, nc, n2, nnz, Fi, Fo, el = s["nS"], s["E"], s["nc"], s["n_next"], s["nnz"], s["F_in"], s["F_out"], s["elt"]
        add = lambda k, b: alg.__setitem__(k, alg.get(k, 0.0) + b)
        add("scan_edges", 8 * E + 20 * nS + 8 * nc)
        add("cand_fused", N / 64 + 8 * nc + 20 * nc)
        add("adj_fused", 4 * E + 16 * nS + 4 * nS + 20 * nnz)
        add("aggregate", n2 * Fi * el + 8 * nnz + 4 * (nS + 1) + 4 * nS * Fi)
        add("layer_gemm", 4 * (nS * Fi + Fi * Fo + nS * Fo))
        flops += 2.0 * nS * Fi * Fo
    kernels = {}
    for k, (ms, cnt) in sorted(prof.items(), key=lambda kv: -kv[1][0]):
        kernels[k] = dict(avg_us=ms / cnt * 1e3, launches_per_step=cnt / args.steps, ms_per_step=ms / args.steps)
        if alg.get(k):
            kernels[k]["alg_GBps"] = alg[k] / (ms * 1e-3) / 1e9
    kernels["layer_gemm"]["TFLOPs"] = flops / (prof["layer_gemm"][0] * 1e-3) / 1e12
    dominant = next(iter(kernels))
    if dominant == "layer_gemm":
        ach = kernels[dominant]["TFLOPs"]
        roofline = dict(bound="mfma", kernel=dominant, achieved=ach, peak=MFMA_F32_PEAK_TFLOPS, unit="TFLOP/s",
                        frac=ach / MFMA_F32_PEAK_TFLOPS, traffic=None)
    else:
        ach = kernels[dominant].get("alg_GBps", 0.0)
        roofline = dict(bound="hbm", kernel=dominant, achieved=ach, peak=HBM_PEAK_GBS, unit="GB/s",
                        frac=ach / HBM_PEAK_GBS, traffic=None)
    roofline["avg_launch_us"] = kernels[dominant]["avg_us"]
    roofline["alg_bytes_per_launch"] = alg.get(dominant, 0.0) / max(prof[dominant][1], 1)

    tot = lambda key: sum(s[key] for s in sizes) / args.steps
    sampled_edges_per_step = tot("nnz")
    value = sampled_edges_per_step / (ms_per_step * 1e-3)

    cpu_baseline = None
    if not args.no_cpu_baseline:
        import chain
        n_cpu = 2
        t0 = time.perf_counter()
        cpu_nnz = 0
        for it in range(args.warmup, args.warmup + n_cpu):
            osteps = chain.oracle_chain(g, X, Ws, batches[it], cfg.skew, B, seed, it, bf16)
            cpu_nnz += sum(o.sm.adj_nnz for o in osteps)
            if it == args.warmup:   # spot check: the GPU step of the same batch drew the same nodes
                want = [s for s in sizes if True][:M]
                for l, o in enumerate(osteps):
                    assert want[l]["n_next"] == o.sm.n_next and want[l]["nnz"] == o.sm.adj_nnz
                    assert want[l]["remote"] == o.rc.remote_total
        cpu_s = time.perf_counter() - t0
        cpu_baseline = dict(value=cpu_nnz / cpu_s, unit="sampled edges/s", cores=1, kind="oracle",
                            sample=f"{n_cpu} whole steps of the same workload ({cpu_s:.1f} s)",
                            ms_per_step=cpu_s / n_cpu * 1e3)

    out = dict(
        metric="sampled-aggregation HBM GB/s + sampled edges/s per GCN layer; step time",
        value=value, unit="sampled edges/s", n_gpus=1, steps=args.steps, warmup=args.warmup,
        ms_per_step=ms_per_step, higher_is_better=True, scaling="weak", vs_baseline=None,
        dtype="bf16 features, f32 accumulate" if bf16 else "f32", data="synthetic",
        config=dict(workload=f"{cfg.name}: N={g.n_nodes}, nnz={g.nnz}, {cfg.n_parts} partitions, batch {cfg.batch}, "
                             f"{B} samples/layer, {M} layers {dims}, skew {cfg.skew}",
                    per_step=dict(edges_scanned=tot("E"), candidates=tot("nc"), sampled_nodes=tot("n_next"),
                                  sampled_edges=sampled_edges_per_step, remote_nodes=tot("remote"))),
        aggregate_GBps=kernels.get("aggregate", {}).get("alg_GBps"),
        gemm_TFLOPs=kernels["layer_gemm"]["TFLOPs"],
        scanned_edges_per_s=tot("E") / (ms_per_step * 1e-3),
        roofline=roofline, cpu_baseline=cpu_baseline, kernels=kernels)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
