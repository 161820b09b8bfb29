#!/usr/bin/env python3
"""Benchmark of one partition's sampled mini-batch step on one MI355X.

A step = the whole hot path over one batch of synthetic input: for every GCN layer, top-down,
csgs_build_probs -> csgs_sample_layer -> csgs_remote_count; then, bottom-up, csgs_aggregate ->
csgs_layer_gemm.  Inputs are resident in HBM before the timed region.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config large] [--scale S] [--instances 8]

The timed schedule handles several consecutive mini-batches per library call (--instances), samples
such groups on two streams and computes their layers on a third; every step still does all of its
work.  Afterwards every kernel is timed launch by launch, inside that schedule and alone on one
stream; the roofline figures come from the durations alone.

Besides the named workload the default run also times a scaled-up variant of it (batch and samples
per layer x16, same graph): the named batch moves only a few MB per kernel, which no kernel can
turn into a large fraction of 8 TB/s within its launch latency, so the scaled run is where the
kernels' bandwidth / MFMA efficiency shows.  It is reported under "scaled", never as `value`.
"""
import argparse
import dataclasses
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

HBM_PEAK_GBS = 8000.0
MFMA_F64_PEAK_TFLOPS = 78.6     # the layer GEMM accumulates on the fp64 matrix cores


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def algorithmic_bytes(s, N):
    """Bytes each kernel must move for one layer step of the given sizes (each item once)."""
    nS, E, nc, n2, nnz, Fi, Fo, el, B = (s[k] for k in ("nS", "E", "nc", "n_next", "nnz", "F_in", "F_out", "elt", "B"))
    agg = n2 * Fi * el + 8 * nnz + 4 * (nS + 1) + 4 * nS * Fi
    return {
        "row_prefix": 28 * nS,                              # S, two row pointers, prefix + start written
        "scan_edges": 8 * E + 16 * nS + 8 * nc,             # col + val per edge, row slices, accumulators
        "cand_partials": N / 64 + 8 * nc,                   # flags, accumulators read
        "cand_emit": N / 64 + 8 * nc + 20 * nc,             # the same again, id + weight + cdf written
        "draw": 12 * B,                                     # cdf probes are cache traffic
        "hits_fused": nc / 8 + 36 * n2,                     # position bitmap, per hit: count, 2 cdf, id, 4 outputs
        "adj_fused": 4 * E + 16 * nS + 4 * nS + 20 * nnz,   # col per edge, row slices, row pointers, kept edges
        "remote_count": 12 * n2,
        "aggregate": agg,
        "layer_gemm": 4 * (nS * Fi + Fi * Fo + nS * Fo),
        "gather_rows": 0.0,                                 # filled in by the caller (remote rows, bottom layer only)
    }


class Workload:
    def __init__(self, cfg, g, dg, Xd, dev, n_batches, torch, pipeline, synth, csgs, n_samplers=1, n_inst=1, batch_compute=False,
                 fused=None, n_comp=1):
        self.cfg, self.g, self.dg, self.Xd, self.dev = cfg, g, dg, Xd, dev
        self.n_comp = n_comp    # streams for the layer compute: buffer set k is computed on stream k % n_comp
        self.fused = fused      # None: csgs_aggregate + csgs_layer_gemm; "h" / "hz": csgs_layer_forward where it takes the width
        self.torch, self.pipeline, self.csgs = torch, pipeline, csgs
        self.bf16 = cfg.feat_dtype == "bf16"
        self.dims = synth.layer_dims(cfg)
        self.M = len(self.dims)
        self.B = cfg.samples
        self.seed = 1234 + cfg.seed
        self.Ws = [synth.glorot_uniform(fi, fo, cfg.seed) for fi, fo in self.dims]
        self.batches = [synth.make_batch(g, cfg.batch, cfg.seed, it) for it in range(n_batches)]
        self.X_local = Xd[g.local_lo:g.local_hi]
        self.Wd = [torch.from_numpy(W).to(dev) for W in self.Ws]
        self.Sd = [torch.from_numpy(b).to(dev) for b in self.batches]
        M, B, dims = self.M, self.B, self.dims
        nS_max = max(len(self.batches[0]), B)
        self.n_samplers, self.n_inst = n_samplers, n_inst
        adj_cap = int(min(g.nnz, 16_000_000))
        # one mini-batch per call: the one-stream (latency) measurement and the backward pass
        self.lbs1 = [pipeline.LayerBuffers(nS_max, B, g.n_nodes, adj_cap, dg.n_parts, dev) for _ in range(M)]
        self.ws1 = pipeline.Workspace(g.n_nodes, nS_max, B, g.nnz, dev)
        # the timed schedule: n_inst mini-batches per sampling call.  Sets of sampling outputs: while the
        # layers of one group of batches are computed from one set, later groups are sampled into the others
        self.n_sets = 2 * n_samplers
        self.lb_sets = [[pipeline.LayerBuffers(nS_max, B, g.n_nodes, adj_cap, dg.n_parts, dev, n_inst=n_inst) for _ in range(M)]
                        for _ in range(self.n_sets)]
        self.wss = [pipeline.Workspace(g.n_nodes, nS_max, B, g.nnz, dev, n_inst=n_inst, inst_stride=self.lb_sets[0][0].stride)
                    for _ in range(n_samplers)]   # one per sampling stream
        self.lb_inst = [[[lb.inst(k) for lb in lbs] for k in range(n_inst)] for lbs in self.lb_sets]   # [set][instance][layer]
        self.lbs = self.lbs1
        self.overlap = None
        self.use_graphs = True
        self.one_stream = False  # --one-stream: the timed schedule without any overlap (what the profiler summaries are made with)
        self.direct = False     # issue the timed schedule call by call (for per-dispatch timing, which a graph replay cannot carry)
        self.Zs = [torch.empty((nS_max, dims[M - 1 - l][0]), dtype=torch.float32, device=dev) for l in range(M)]
        self.Hs = [torch.empty((nS_max, dims[M - 1 - l][1]), dtype=torch.float32, device=dev) for l in range(M)]
        self.elt = 2 if self.bf16 else 4
        self.staged = torch.zeros((B, Xd.shape[1]), dtype=Xd.dtype, device=dev)   # sampled remote feature rows
        # all instances of a group through the same compute launches: per-instance Z, H and staged rows
        self.batch_compute = batch_compute and n_inst > 1
        if self.batch_compute:      # one set of these per compute stream
            self.ZsK_c = [[torch.empty((n_inst, nS_max, dims[M - 1 - l][0]), dtype=torch.float32, device=dev) for l in range(M)] for _ in range(n_comp)]
            self.HsK_c = [[torch.empty((n_inst, nS_max, dims[M - 1 - l][1]), dtype=torch.float32, device=dev) for l in range(M)] for _ in range(n_comp)]
            self.stagedK_c = [torch.zeros((n_inst, B, Xd.shape[1]), dtype=Xd.dtype, device=dev) for _ in range(n_comp)]
            self.ZsK, self.HsK, self.stagedK = self.ZsK_c[0], self.HsK_c[0], self.stagedK_c[0]

    def enqueue_sampling(self, S0, it, lbs, ws):
        """Top-down sampling calls on the current stream, for one mini-batch or, when `ws` and `lbs`
        hold several instances, for that many at once (instance k: the rows at S0 + k strides, iteration
        it + k); `it` is a number or a device uint64 tensor."""
        cfg, M, B, pipeline = self.cfg, self.M, self.B, self.pipeline
        it_num, it_dev = (0, it) if hasattr(it, "data_ptr") else (it, None)
        for l in range(M):
            # layers after the first take the rows the previous layer's sampler prepared (S None)
            pipeline.sample_step(self.dg, ws, S0 if l == 0 else None, cfg.skew, B, self.seed, it_num, l, lbs[l],
                                 want_q=False, iter_dev=it_dev)

    def enqueue_compute(self, lbs, n0):
        """Staging of the sampled remote rows (stands in for their exchange) and the bottom-up layer
        compute of one mini-batch on the current stream."""
        M, B, pipeline = self.M, self.B, self.pipeline
        pipeline.stage_remote_rows(lbs[M - 1], self.Xd, self.staged)
        H = None
        for l in range(M - 1, -1, -1):
            nS = n0 if l == 0 else B
            nS_dev = None if l == 0 else lbs[l - 1].n_next
            Z, Hn = self.Zs[l][:nS], self.Hs[l][:nS]
            if l == M - 1:
                pipeline.compute_step(lbs[l], nS, self.X_local, self.staged, True, False, self.Wd[0], Z, Hn, nS_dev=nS_dev, fused=self.fused)
            else:
                pipeline.compute_step(lbs[l], nS, H, None, False, True, self.Wd[M - 1 - l], Z, Hn, nS_dev=nS_dev, fused=self.fused)
            H = Hn
        return H

    def enqueue_compute_group(self, lbs, n0, kk=None, c=0):
        """The same for the first kk instances (default: all) of a buffer set in the same launches (the _n
        forms of the calls), into the Z / H / staged-row buffers of compute stream c."""
        M, B, pipeline = self.M, self.B, self.pipeline
        kk = self.n_inst if kk is None else kk
        nb = lambda t: t.stride(0) * t.element_size()
        ZsK, HsK, stagedK = self.ZsK_c[c], self.HsK_c[c], self.stagedK_c[c]
        pipeline.stage_remote_rows(lbs[M - 1], self.Xd, stagedK[0], out_stride=nb(stagedK), n_inst=kk)
        for l in range(M - 1, -1, -1):
            nS = n0 if l == 0 else B
            nS_dev = None if l == 0 else lbs[l - 1].n_next
            Z, H = ZsK[l], HsK[l]
            if l == M - 1:
                pipeline.compute_step(lbs[l], nS, self.X_local, stagedK[0], True, False, self.Wd[0], Z[0, :nS], H[0, :nS],
                                      nS_dev=nS_dev, strides=(0, nb(stagedK), nb(Z), nb(H)), n_inst=kk, fused=self.fused)
            else:
                pipeline.compute_step(lbs[l], nS, HsK[l + 1][0, :B], None, False, True, self.Wd[M - 1 - l], Z[0, :nS], H[0, :nS],
                                      nS_dev=nS_dev, strides=(nb(HsK[l + 1]), 0, nb(Z), nb(H)), n_inst=kk, fused=self.fused)
        return HsK[0][kk - 1, :n0]

    def prepare_backward(self):
        """Buffers for the gradients of every layer (dW, dZ, dH_prev, scratch), sized for the capacities."""
        torch, csgs, M, B, dims = self.torch, self.csgs, self.M, self.B, self.dims
        dev, n0 = self.dev, self.Sd[0].numel()
        i8 = lambda nbytes: torch.empty(max(nbytes, 256) // 8 + 32, dtype=torch.int64, device=dev)
        self.bw = []
        for l in range(M):
            K, N = dims[M - 1 - l]
            cap = n0 if l == 0 else B
            self.bw.append(dict(
                cap=cap, dW=torch.empty((K, N), device=dev), dZ=torch.empty((cap, K), device=dev),
                dH=torch.empty((B, K), device=dev) if l < M - 1 else None,
                sw=i8(csgs.csgs_layer_gemm_grad_w_scratch_bytes(cap, K, N)),
                sa=i8(csgs.csgs_aggregate_grad_scratch_bytes(B, self.lbs1[l].adj_col.numel())) if l < M - 1 else None))
        g = torch.Generator(device="cpu").manual_seed(5)
        self.G_top = torch.randn((n0, dims[0][1] if M == 1 else dims[M - 1][1]), generator=g).to(dev)

    def backward(self):
        """Gradients of all layers for the batch whose forward pass is in lbs1 / Zs / Hs: top layer
        first, each layer's dH_prev is the next one's dL/dH; row counts stay on the device."""
        csgs, M, B, lbs = self.csgs, self.M, self.B, self.lbs1
        G = self.G_top
        for l in range(M):
            bw, lb = self.bw[l], lbs[l]
            nS_dev = None if l == 0 else lbs[l - 1].n_next
            Z, W = self.Zs[l][:bw["cap"]], self.Wd[M - 1 - l]
            csgs.csgs_layer_gemm_grad_w(Z, G, bw["dW"], bw["sw"], M_dev=nS_dev)
            csgs.csgs_layer_gemm_grad_z(G, W, bw["dZ"], M_dev=nS_dev)
            if l < M - 1:
                csgs.csgs_aggregate_grad(lb.adj_rowptr[:bw["cap"] + 1], lb.adj_col, lb.adj_val, lb.n_next, bw["dZ"],
                                         self.Hs[l + 1][:B], bw["dH"], bw["sa"], nS_dev=nS_dev)
                G = bw["dH"]

    def measure_backward(self, steps):
        """Backward pass alone, back to back on one stream, after one forward step; then per-kernel times."""
        torch, csgs = self.torch, self.csgs
        self.prepare_backward()
        self.step(0)
        for _ in range(3):
            self.backward()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            self.backward()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) / steps * 1e3
        csgs.csgs_profile_enable(True)
        for _ in range(steps):
            self.backward()
        torch.cuda.synchronize()
        csgs.csgs_profile_enable(False)
        prof = csgs.csgs_profile_collect()
        sizes = [int(self.Sd[0].numel())] + [int(self.lbs1[l].n_next.item()) for l in range(self.M - 1)]
        flops = sum(4.0 * sizes[l] * self.dims[self.M - 1 - l][0] * self.dims[self.M - 1 - l][1] for l in range(self.M))
        gemm_ms = sum(prof[k][0] for k in ("gemm_grad_z", "gemm_grad_w", "gemm_grad_w_reduce") if k in prof)
        return dict(ms_per_step=ms, gemm_TFLOPs=flops * steps / (gemm_ms * 1e-3) / 1e12,
                    kernels={k: dict(avg_us=round(v[0] / v[1] * 1e3, 3), launches_per_step=v[1] / steps)
                             for k, v in sorted(prof.items(), key=lambda kv: -kv[1][0])})

    def prepare_overlap(self, rem=0):
        """Streams, events and, per buffer set, the library calls of a group of n_inst mini-batches
        captured into two HIP graphs (sampling of all of them at once, layer compute one after the
        other), and the same for a last, smaller group of `rem` mini-batches when the step count is
        no multiple of n_inst (same buffers, fewer instances per call).  What differs from replay to
        replay goes through device memory: the set's iteration numbers select its batches from the
        resident batch table, and the sampling graph advances them itself.  A kernel launch costs the
        host 4-5 us, so launching a step's kernels one by one cannot keep three streams fed; a replay
        is one call."""
        torch, K, dev = self.torch, self.n_inst, self.dev
        samplers = [torch.cuda.Stream() for _ in range(self.n_samplers)]
        s_comps = [torch.cuda.Stream() for _ in range(self.n_comp)]
        self.S_all = torch.stack(self.Sd)        # all batches, resident: [n_batches, batch]
        n0 = self.Sd[0].numel()
        sizes_k = [K] + ([rem] if 0 < rem < K else [])
        sets = []
        for k in range(self.n_sets):
            s_samp = samplers[k % self.n_samplers]
            c, s_comp = k % self.n_comp, s_comps[k % self.n_comp]
            lbs, ws = self.lb_sets[k], self.wss[k % self.n_samplers]
            lb0 = lbs[0]
            # first-layer rows of all instances: the S0 arrays of the set, one stride apart
            S0_all = torch.as_strided(lb0.S0, (K, n0), (lb0.stride // 4, 1))
            idx = torch.arange(K, dtype=torch.int64, device=dev)      # iteration number of every instance
            tmp = torch.zeros((K, n0), dtype=self.S_all.dtype, device=dev)

            def fill(kk, idx=idx, tmp=tmp, S0_all=S0_all, lb0=lb0):
                if K == 1:      # straight into the row array
                    torch.index_select(self.S_all, 0, idx, out=lb0.S0[:n0].view(1, -1))
                else:
                    torch.index_select(self.S_all, 0, idx[:kk], out=tmp[:kk])   # the batches of these iterations
                    S0_all[:kk].copy_(tmp[:kk])

            def sample(kk=K, idx=idx, lbs=lbs, ws=ws, lb0=lb0, fill=fill):
                fill(kk)
                ws.desc.n_inst = kk       # instances of this call (the descriptor is read when the call is made)
                self.enqueue_sampling(lb0.S0[:n0], idx, lbs, ws)      # the library reads idx[0]; instance k uses idx[0] + k
                ws.desc.n_inst = K

            def compute(kk=K, k=k, lbs=lbs, c=c):
                if self.batch_compute:
                    return self.enqueue_compute_group(lbs, n0, kk, c)
                H = None
                for lk in self.lb_inst[k][:kk]:
                    H = self.enqueue_compute(lk, n0)
                return H

            # one eager pass on the streams the graphs will run on, then capture
            torch.cuda.synchronize()
            with torch.cuda.stream(s_samp):
                sample()
            torch.cuda.synchronize()
            with torch.cuda.stream(s_comp):
                compute()
            torch.cuda.synchronize()
            graphs = {}
            if self.use_graphs:
                try:
                    for kk in sizes_k:
                        g_samp, g_comp = torch.cuda.CUDAGraph(), torch.cuda.CUDAGraph()
                        with torch.cuda.graph(g_samp, stream=s_samp):
                            sample(kk)
                            if kk == K:
                                idx.add_(K * self.n_sets)     # the next replay of this set is n_sets groups later
                        with torch.cuda.graph(g_comp, stream=s_comp):
                            compute(kk)
                        graphs[kk] = (g_samp, g_comp)
                except Exception as e:      # said out loud and recorded in the JSON line; the calls are then issued one by one
                    log(f"graph capture failed ({e!r}); launching the calls directly")
                    self.use_graphs = False
                    graphs = {}
            torch.cuda.synchronize()
            H_of = lambda kk, c=c: self.HsK_c[c][0][kk - 1, :n0] if self.batch_compute else self.Hs[0][:n0]
            sets.append(dict(idx=idx, graphs=graphs, sample_fn=sample, compute_fn=compute, H_of=H_of,
                             s_samp=s_samp, s_comp=s_comp, samp_done=torch.cuda.Event(), comp_done=torch.cuda.Event(), used=False))
        self.it_host = torch.arange(0, len(self.Sd), dtype=torch.int64, device=dev)   # iteration numbers, resident
        self.graph_it = [None] * self.n_sets     # first iteration number each set's counters hold for its next replay
        self.overlap = dict(sets=sets, s_comp=s_comps[0])

    def group(self, it0, kk=None, seq=None):
        """Mini-batches it0 .. it0 + kk - 1 (kk = n_inst unless it is the one smaller group), enqueued without the
        host waiting for anything; seq: the group's number in the sequence of groups (default it0 // n_inst), which
        picks its buffer set and streams.  Their sampling (top-down)
        is ONE sequence of library calls over kk instances; consecutive groups go round-robin to
        n_samplers streams, each with its own workspace.  The layer compute (bottom-up) of all batches
        runs in batch order on one more stream; events tie a group's compute to its sampling and a
        buffer set's reuse to the compute that read it.  This is how a training loop runs its sampler
        ahead: sampling does not depend on the model weights, the compute of consecutive batches does.
        Every step still does all of its work."""
        torch, K = self.torch, self.n_inst
        kk = K if kk is None else kk
        k = (it0 // K if seq is None else seq) % self.n_sets
        st = self.overlap["sets"][k]
        s_comp = self.overlap["s_comp"] if self.one_stream else st["s_comp"]
        g_samp, g_comp = st["graphs"].get(kk, (None, None))
        if self.one_stream:     # everything in order on the compute stream: every kernel has the device to itself
            with torch.cuda.stream(s_comp):
                st["idx"][:kk].copy_(self.it_host[it0:it0 + kk], non_blocking=True)
                if g_samp is not None:
                    g_samp.replay()
                    g_comp.replay()
                else:
                    st["sample_fn"](kk)
                    st["compute_fn"](kk)
                self.graph_it[k] = None
            return st["H_of"](kk)
        with torch.cuda.stream(st["s_samp"]):
            if st["used"]:
                st["s_samp"].wait_event(st["comp_done"])     # the set is free once the batches sampled into it were computed
            direct = g_samp is None or self.direct     # call by call instead of a graph replay
            if direct or kk != K or self.graph_it[k] != it0:   # (re)seat the set's counters; consecutive full replays advance them
                st["idx"][:kk].copy_(self.it_host[it0:it0 + kk], non_blocking=True)
            if not direct:
                g_samp.replay()
                self.graph_it[k] = it0 + K * self.n_sets if kk == K else None
            else:
                st["sample_fn"](kk)
                self.graph_it[k] = None
            st["samp_done"].record(st["s_samp"])
        with torch.cuda.stream(s_comp):
            s_comp.wait_event(st["samp_done"])
            if g_comp is not None and not self.direct:
                g_comp.replay()
            else:
                st["compute_fn"](kk)
            st["comp_done"].record(s_comp)
        st["used"] = True
        return st["H_of"](kk)

    def theorem1_sweep(self, Ds=(4.0, 8.0, 16.0, 32.0), it=0):
        """One mini-batch sampled with the skew chosen on the device by Theorem 1 (Eq. 12) for each D of the
        paper's sweep (Section 5.2): per layer the skew that was used and the sampled remote nodes, and for the
        bottom layer (whose remote nodes are the feature vectors that would be transferred) their expectation
        sum_{j in R} p_j (Eq. 4 with Eq. 8) from the distribution the call wrote."""
        torch, pipeline, M, B = self.torch, self.pipeline, self.M, self.B
        out = []
        for D in Ds:
            for l in range(M):
                pipeline.sample_step(self.dg, self.ws1, self.Sd[it] if l == 0 else None, 4096.0, B, self.seed, it, l, self.lbs1[l],
                                     want_q=False, auto_D=D)
            torch.cuda.synchronize()
            layers = []
            for l in range(M):
                lb, st = self.lbs1[l], self.lbs1[l].stats_host()
                assert int(lb.status.item()) == 0
                layers.append(dict(layer=l, skew=st.skew_fx / 16.0, candidates=st.n_cand, remote_candidates=st.n_remote,
                                   sampled_nodes=int(lb.n_next.item()), remote_nodes=int(lb.remote_total.item())))
            lb, st = self.lbs1[M - 1], self.lbs1[M - 1].stats_host()
            cdf = lb.cdf[:st.n_cand].to(torch.float64)
            q = torch.diff(cdf, prepend=cdf.new_zeros(1)) / float(st.total)
            ids = lb.cand_id[:st.n_cand]
            rem = (ids < self.g.local_lo) | (ids >= self.g.local_hi)
            expect = float((-torch.expm1(B * torch.log1p(-q[rem]))).sum().item())
            out.append(dict(D=D, bottom_layer_remote_nodes=layers[-1]["remote_nodes"], bottom_layer_expected_remote_nodes=expect,
                            layers=layers))
        return out

    def sizes_of(self, lbs, n0, sizes):
        M, B = self.M, self.B
        for l in range(M):
            st = lbs[l].stats_host()
            sizes.append(dict(layer=l, nS=n0 if l == 0 else int(lbs[l - 1].n_next.item()), E=st.edges_scanned,
                              nc=st.n_cand, B=B, n_next=int(lbs[l].n_next.item()), nnz=int(lbs[l].adj_nnz.item()),
                              remote=int(lbs[l].remote_total.item()), F_in=self.dims[M - 1 - l][0],
                              F_out=self.dims[M - 1 - l][1], elt=self.elt if l == M - 1 else 4,
                              status=int(lbs[l].status.item())))

    def step(self, it, sizes=None):
        """One whole mini-batch on the current stream, one instance per call, enqueued without the
        host waiting for anything: each layer's row count stays on the device (the n_dev
        arguments), launches are sized for the capacities."""
        n0 = self.Sd[it].numel()
        self.enqueue_sampling(self.Sd[it], it, self.lbs1, self.ws1)
        H = self.enqueue_compute(self.lbs1, n0)
        if sizes is not None:
            self.torch.cuda.synchronize()
            self.sizes_of(self.lbs1, n0, sizes)
        return H

    def measure(self, steps, warmup, serial=True):
        """Timed region: exactly `steps` steps in groups of n_inst mini-batches, the first group smaller
        when n_inst does not divide them (warmup is a multiple of n_inst).  Then the full groups again,
        launched call by call with every kernel launch bracketed by HIP events (recorded on the launch
        stream): every launch these passes time handles n_inst mini-batches, whatever `steps` is."""
        torch, csgs, K = self.torch, self.csgs, self.n_inst
        assert steps >= K and warmup % K == 0 and len(self.Sd) >= steps + warmup
        n0 = self.Sd[0].numel()
        # the one smaller group (when K does not divide the steps) goes first: the compute stream, idle until the first
        # group is sampled, then starts sooner, and what the region ends with is a full group's compute either way
        rem = steps % K
        chunks = ([(warmup, rem)] if rem else []) + [(it0, K) for it0 in range(warmup + rem, warmup + steps, K)]
        full = [c for c in chunks if c[1] == K]
        # (1) one stream, one mini-batch per call, steps back to back: the latency of a step
        serial_ms, h_serial = None, None
        if serial:
            for it in range(warmup):
                self.step(it)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for it in range(warmup, warmup + steps):
                H = self.step(it)
            torch.cuda.synchronize()
            serial_ms = (time.perf_counter() - t0) / steps * 1e3
            h_serial = H.clone()
        # (2) the timed region proper: the same steps, n_inst per sampling call, sampling and compute overlapped
        if self.overlap is None:
            self.prepare_overlap(rem=steps % K)
        for it0 in range(0, warmup, K):
            self.group(it0)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for seq, (it0, kk) in enumerate(chunks):
            H = self.group(it0, kk, seq)
        enqueue_ms = (time.perf_counter() - t0) / steps * 1e3     # host time to enqueue a step (no waiting in it)
        torch.cuda.synchronize()
        ms_per_step = (time.perf_counter() - t0) / steps * 1e3
        if serial:
            assert torch.equal(H, h_serial), "the timed schedule must give the one-stream result bit for bit"
        assert all(int(lb.status.item()) == 0 for set_ in self.lb_inst for lk in set_ for lb in lk), \
            "a status bit was set in the timed run"
        log(f"host enqueue {enqueue_ms:.3f} ms/step; " + (f"one stream, one batch per call {serial_ms:.3f} ms/step; " if serial else "") +
            f"{K} batches per sampling call" + (f" (first group {chunks[0][1]})" if chunks[0][1] != K else "") + ", " +
            ("everything in order on one stream" if self.one_stream else "sampling and compute overlapped") +
            f" {ms_per_step:.3f} ms/step")
        # (3) how long the kernels take inside the timed schedule, beside the kernels of the other streams: the full
        # groups on the same streams, launched call by call so that every dispatch carries its pair of events (the
        # host stays well ahead of the device)
        prof_sched = {}
        n_rep = max(1, -(-16 // len(full)))      # at least 16 groups in each per-kernel pass
        if not self.one_stream:
            csgs.csgs_profile_enable(True)
            self.direct = True
            for _ in range(n_rep):
                for it0, kk in full:
                    self.group(it0, kk)
            torch.cuda.synchronize()
            self.direct = False
            csgs.csgs_profile_enable(False)
            prof_sched = csgs.csgs_profile_collect()
        # (4) the full groups again on one stream, back to back without the host reading anything in between (the device
        # stays busy as in the timed region), at least 16 groups: every kernel's own duration with the device to itself
        # -- what the roofline figures are taken from.  Then once more, untimed, with a wait after every group to read
        # the sizes of every step (they depend on the iteration numbers only)
        st0 = self.overlap["sets"][0]
        st0["idx"].copy_(self.it_host[full[0][0]:full[0][0] + K])
        st0["sample_fn"]()
        st0["compute_fn"]()
        torch.cuda.synchronize()
        csgs.csgs_profile_enable(True)
        for _ in range(n_rep):
            for it0, kk in full:
                st0["idx"].copy_(self.it_host[it0:it0 + K], non_blocking=True)
                st0["sample_fn"]()
                st0["compute_fn"]()
        torch.cuda.synchronize()
        csgs.csgs_profile_enable(False)
        samples = csgs.csgs_profile_samples()
        prof = csgs.csgs_profile_collect()
        sizes = []
        for it0, kk in full:
            st0["idx"].copy_(self.it_host[it0:it0 + K])
            st0["sample_fn"]()
            st0["compute_fn"]()
            torch.cuda.synchronize()
            for lk in self.lb_inst[0]:
                self.sizes_of(lk, n0, sizes)
        self.graph_it[0] = None
        assert all(s["status"] == 0 for s in sizes), "a status bit was set"
        sizes_once = sizes
        sizes = sizes * n_rep       # what the timed launches of pass (4) processed
        steps = n_rep * len(full) * K       # the steps the per-kernel passes covered: what the averages below are over
        alg, flops, flops_fused = {}, 0.0, 0.0
        one_kernel = lambda s: bool(self.fused) and bool(csgs.lib().csgs_layer_forward_supported(s["F_in"], 0, s["F_in"], s["F_in"]))
        for s in sizes:
            ab = algorithmic_bytes(s, self.g.n_nodes)
            if one_kernel(s):   # Z stays on the chip (or is written once, never read back), W and H as in the product
                z = 4.0 * s["nS"] * s["F_in"]
                ab["layer_forward"] = ab.pop("aggregate") - z + ab.pop("layer_gemm") - z + (z if self.fused == "hz" else 0.0)
                flops_fused += 2.0 * s["nS"] * s["F_in"] * s["F_out"]
            else:
                flops += 2.0 * s["nS"] * s["F_in"] * s["F_out"]
            for k, b in ab.items():
                alg[k] = alg.get(k, 0.0) + b
            if s["layer"] == self.M - 1:    # staged remote rows: read once, written once
                alg["gather_rows"] = alg.get("gather_rows", 0.0) + 2.0 * s["remote"] * s["F_in"] * s["elt"]
        kernels = {}
        for k, (ms, cnt) in sorted(prof.items(), key=lambda kv: -kv[1][0]):
            if k == "fill_zero":
                continue
            kernels[k] = dict(avg_us=ms / cnt * 1e3, launches_per_step=cnt / steps, ms_per_step=ms / steps,
                              alg_bytes_per_launch=alg.get(k, 0.0) / cnt)
            if alg.get(k):
                kernels[k]["alg_GBps"] = alg[k] / (ms * 1e-3) / 1e9
            if k in prof_sched:
                kernels[k]["in_schedule_us"] = prof_sched[k][0] / prof_sched[k][1] * 1e3
            sm = sorted(samples.get(k, []))
            if sm:      # launch by launch: median and the 10th / 90th percentile, in us
                pick = lambda f: sm[min(len(sm) - 1, int(f * len(sm)))] * 1e3
                kernels[k].update(p10_us=pick(0.10), p50_us=pick(0.50), p90_us=pick(0.90))
        agg_GBps = gemm_TF = None
        if "aggregate" in prof:
            agg_GBps = alg["aggregate"] / (prof["aggregate"][0] * 1e-3) / 1e9
        if "layer_gemm" in prof:
            gemm_TF = flops / (prof["layer_gemm"][0] * 1e-3) / 1e12
            kernels["layer_gemm"]["TFLOPs"] = gemm_TF
            kernels["layer_gemm"]["flop_per_launch"] = flops / prof["layer_gemm"][1]
        if "layer_forward" in prof:
            kernels["layer_forward"]["TFLOPs"] = flops_fused / (prof["layer_forward"][0] * 1e-3) / 1e12
            kernels["layer_forward"]["flop_per_launch"] = flops_fused / prof["layer_forward"][1]
        tot = lambda key: sum(s[key] for s in sizes) / steps
        per_step = dict(edges_scanned=tot("E"), candidates=tot("nc"), sampled_nodes=tot("n_next"),
                        sampled_edges=tot("nnz"), remote_nodes=tot("remote"))
        # the same per layer (layer 0 = the batch's own layer, the last one reads the feature table)
        per_layer = []
        for l in range(self.M):
            ls = [x for x in sizes if x["layer"] == l]
            avg = lambda key: round(sum(x[key] for x in ls) / len(ls), 1)
            per_layer.append(dict(layer=l, rows=avg("nS"), edges_scanned=avg("E"), candidates=avg("nc"), sampled_nodes=avg("n_next"),
                                  sampled_edges=avg("nnz"), remote_nodes=avg("remote"), F_in=ls[0]["F_in"], F_out=ls[0]["F_out"]))
        per_step["per_layer"] = per_layer
        return dict(ms_per_step=ms_per_step, serial_ms_per_step=serial_ms, graphs=self.use_graphs, kernels=kernels, per_step=per_step, sizes=sizes_once, sizes_it=full[0][0],
                    aggregate_GBps=agg_GBps, gemm_TFLOPs=gemm_TF, smaller_group=chunks[0][1] if chunks[0][1] != K else None)


MFMA_F32_PEAK_TFLOPS = 157.3    # the fp32 matrix peak, for comparison: the GEMM's inputs and outputs are fp32


def roofline_of(kernels, name, traffic, k_inst):
    """Roofline object of one kernel.  traffic: (bytes per launch by kernel name or None, where from / why not)."""
    k = kernels[name]
    if name in ("layer_gemm", "layer_forward"):
        r = dict(bound="mfma", kernel=name, achieved=k["TFLOPs"], peak=MFMA_F64_PEAK_TFLOPS, unit="TFLOP/s",
                 frac=k["TFLOPs"] / MFMA_F64_PEAK_TFLOPS, alg_per_launch=k["flop_per_launch"],
                 peak_is="fp64 matrix cores (the kernel multiplies and accumulates in double)",
                 frac_of_fp32_matrix_peak=k["TFLOPs"] / MFMA_F32_PEAK_TFLOPS)
    else:
        a = k.get("alg_GBps", 0.0)
        r = dict(bound="hbm", kernel=name, achieved=a, peak=HBM_PEAK_GBS, unit="GB/s", frac=a / HBM_PEAK_GBS,
                 alg_per_launch=k["alg_bytes_per_launch"])
    table, note = traffic
    r["traffic"] = (table or {}).get(name)
    r["traffic_source"] = note
    r["avg_launch_us"] = k["avg_us"]
    r["mini_batches_per_launch"] = k_inst
    return r


def load_traffic(workload, k_inst, one_kernel=False):
    """HBM bytes per launch and kernel from the committed counter summary profiles/<workload>_step_hbm_traffic.txt
    (<workload>_step_layer_forward_hbm_traffic.txt for the schedule with csgs_layer_forward), if that summary was
    taken with the same number of mini-batches per launch; else (None, why)."""
    path = os.path.join(ROOT, "profiles", f"{workload}_step_{'layer_forward_' if one_kernel else ''}hbm_traffic.txt")
    if not os.path.exists(path):
        return None, f"no counter summary for workload {workload} under profiles/"
    lines = open(path).read().splitlines()
    import re
    m = re.search(r"(\d+) mini-batch(?:es)? per launch", lines[0]) if lines else None
    if not m:
        return None, f"{os.path.basename(path)} does not state its mini-batches per launch"
    if int(m.group(1)) != k_inst:
        return None, f"{os.path.basename(path)} was taken with {m.group(1)} mini-batches per launch, this run uses {k_inst}"
    table, in_table = {}, False
    for ln in lines:
        f = ln.split()
        if f[:1] == ["kernel"]:
            in_table = True
        elif in_table and len(f) == 5:
            table[f[0]] = float(f[4]) * 1e6
        elif in_table and not f:
            break
    return table, f"profiles/{os.path.basename(path)} (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, calibrated on the copy kernel; {k_inst} mini-batches per launch)"


def cpu_model():
    try:
        for ln in open("/proc/cpuinfo"):
            if ln.lower().startswith("model name"):
                return ln.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="large")
    ap.add_argument("--scale", type=int, default=1, help="multiply batch and samples per layer of the main workload")
    ap.add_argument("--samplers", type=int, default=2, help="sampling streams (groups of batches sampled side by side)")
    ap.add_argument("--compute-streams", type=int, default=1, help="streams for the layer compute (consecutive groups round-robin)")
    ap.add_argument("--instances", type=int, default=8, help="mini-batches per library call in the timed schedule (at most)")
    ap.add_argument("--no-batch-compute", action="store_true", help="with --instances K: sample K mini-batches per call but "
                    "compute their layers batch by batch (what a training loop must do: its forward passes depend on "
                    "each other through the weights; the forward passes timed here do not)")
    ap.add_argument("--one-stream", action="store_true", help="time the schedule without overlap: sampling and compute of every "
                    "group in order on one stream (every launch then has the device to itself: what the profiler summaries are made with)")
    ap.add_argument("--no-serial", action="store_true", help="skip the one-stream, one-batch-per-call measurement")
    ap.add_argument("--sweep-instances", default="", help="comma-separated K: also time the schedule with K mini-batches per "
                    "sampling call and report step time and the weight scan's rate under \"instances_sweep\"")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-scaled", action="store_true", help="skip the x16 scaled-up variant")
    ap.add_argument("--no-backward", action="store_true", help="skip the timing of the backward pass")
    ap.add_argument("--no-theorem1", action="store_true", help="skip the sweep of D with the skew chosen by Theorem 1")
    ap.add_argument("--no-layer-compare", action="store_true", help="skip the timing of the other --layer-compute choice")
    ap.add_argument("--layer-compute", default="two", choices=["two", "h", "hz"],
                    help="two: csgs_aggregate + csgs_layer_gemm; h: csgs_layer_forward (Z stays in LDS); hz: the same with Z written as well")
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
        cfg = dataclasses.replace(cfg, batch=cfg.batch * args.scale, samples=cfg.samples * args.scale)
    name = cfg.name if args.scale == 1 else f"{cfg.name}_x{args.scale}"
    bf16 = cfg.feat_dtype == "bf16"
    t0 = time.time()
    g = synth.make_graph(cfg)
    log(f"graph {cfg.name}: N={g.n_nodes} nnz={g.nnz} local=[{g.local_lo},{g.local_hi}) in {time.time() - t0:.1f}s")
    X = synth.make_features(cfg.n_nodes, cfg.feat_dim, cfg.seed)
    dg = pipeline.DeviceGraph(g, dev)
    Xh = synth.to_bf16_bits(X).view(np.int16) if bf16 else X
    Xd = torch.from_numpy(Xh).to(dev)
    fused = None if args.layer_compute == "two" else args.layer_compute
    mk = lambda c, nb, K, fused=fused: Workload(c, g, dg, Xd, dev, nb, torch, pipeline, synth, csgs, n_samplers=args.samplers, n_inst=K,
                                                batch_compute=not args.no_batch_compute, fused=fused, n_comp=args.compute_streams)
    # a step is one mini-batch; the timed schedule handles K of them per call, whatever --steps is: exactly --steps
    # steps are timed, the first group being smaller when K does not divide them, and the per-kernel timing passes
    # (what the roofline figures come from) cover the full groups only.  The (untimed) warm-up is rounded up to a
    # multiple of K
    K = max(1, min(args.instances, args.steps))
    args.warmup = (args.warmup + K - 1) // K * K

    # copy-kernel yardstick (also the known-size kernel for calibrating byte counters)
    cbytes = 512 * 2 ** 20
    ca = torch.zeros(cbytes // 8, dtype=torch.int64, device=dev)
    cb = torch.empty_like(ca)
    for _ in range(3):
        csgs.csgs_calib_copy(cb, ca)
    torch.cuda.synchronize()
    csgs.csgs_profile_enable(True)
    for _ in range(5):
        csgs.csgs_calib_copy(cb, ca)
    torch.cuda.synchronize()
    csgs.csgs_profile_enable(False)
    cms, ccnt = csgs.csgs_profile_collect()["copy"]
    copy_GBps = 2 * cbytes * ccnt / (cms * 1e-3) / 1e9
    del ca, cb
    # atomic-update yardstick: 64-bit adds to random entries of a table as large as the weight accumulators
    table = torch.zeros(g.n_nodes, dtype=torch.int64, device=dev)
    n_upd = 1 << 24
    for _ in range(2):
        csgs.csgs_calib_atomics(table, n_upd)
    torch.cuda.synchronize()
    csgs.csgs_profile_enable(True)
    for _ in range(5):
        csgs.csgs_calib_atomics(table, n_upd)
    torch.cuda.synchronize()
    csgs.csgs_profile_enable(False)
    ams, acnt = csgs.csgs_profile_collect()["atomics"]
    atomic_Gups = n_upd * acnt / (ams * 1e-3) / 1e9
    del table
    # random-lookup yardstick: 8-byte reads of random entries of the same table (the adjacency pass looks up one per edge)
    table = torch.zeros(g.n_nodes, dtype=torch.int64, device=dev)
    lsink = torch.zeros(1 << 22, dtype=torch.int64, device=dev)
    for _ in range(2):
        csgs.csgs_calib_lookups(table, n_upd, lsink)
    torch.cuda.synchronize()
    csgs.csgs_profile_enable(True)
    for _ in range(5):
        csgs.csgs_calib_lookups(table, n_upd, lsink)
    torch.cuda.synchronize()
    csgs.csgs_profile_enable(False)
    lms, lcnt = csgs.csgs_profile_collect()["lookups"]
    lookup_Gps = n_upd * lcnt / (lms * 1e-3) / 1e9
    del table, lsink
    # gather of a known volume: 1 Mi distinct random rows of 256 bytes out of a 1 GiB table through csgs_gather_rows (256 MiB
    # read, 256 MiB written): the non-streaming kernel of known size against which the byte counters' calibration is checked
    gt = torch.zeros((1 << 22, 64), dtype=torch.float32, device=dev)
    gids = torch.randperm(1 << 22, device=dev, generator=torch.Generator(device=dev).manual_seed(7))[:1 << 20].to(torch.int32)
    gout = torch.empty((1 << 20, 64), dtype=torch.float32, device=dev)
    for _ in range(2):
        csgs.csgs_gather_rows(gt, gids, None, gout)
    torch.cuda.synchronize()
    csgs.csgs_profile_enable(True)
    for _ in range(5):
        csgs.csgs_gather_rows(gt, gids, None, gout)
    torch.cuda.synchronize()
    csgs.csgs_profile_enable(False)
    gms, gcnt = csgs.csgs_profile_collect()["gather_rows"]
    gather_GBps = 2 * (1 << 28) * gcnt / (gms * 1e-3) / 1e9
    del gt, gids, gout
    # matrix-core yardstick: the GEMM's instruction (fp64 16 x 16 x 4) back to back from registers, and the
    # GEMM's inner loop (operands from LDS, widened) without its global loads and barriers
    sink = torch.zeros(csgs.CALIB_MFMA_BLOCKS * 256, dtype=torch.float64, device=dev)
    mfma_TF = {}
    for from_lds in (False, True):
        for _ in range(2):
            csgs.csgs_calib_mfma_f64(sink, 256, from_lds)
        torch.cuda.synchronize()
        csgs.csgs_profile_enable(True)
        flops = sum(csgs.csgs_calib_mfma_f64(sink, 256, from_lds) for _ in range(5))
        torch.cuda.synchronize()
        csgs.csgs_profile_enable(False)
        mms, _ = csgs.csgs_profile_collect()["mfma_f64"]
        mfma_TF[from_lds] = flops / (mms * 1e-3) / 1e12
    del sink
    log(f"copy kernel: {copy_GBps:.0f} GB/s (read + write); gather of random 256-byte rows {gather_GBps:.0f} GB/s (read + write); "
        f"random 8-byte lookups {lookup_Gps:.1f} G/s; 64-bit atomic adds to random addresses: {atomic_Gups:.1f} G/s; "
        f"fp64 matrix instructions back to back: {mfma_TF[False]:.1f} TFLOP/s from registers, {mfma_TF[True]:.1f} with operands from LDS")

    N_CPU = 20      # whole steps the oracle is timed on (about 11 s on one core at Large)
    wl = mk(cfg, max(args.steps, 0 if args.no_cpu_baseline else N_CPU) + args.warmup, K)
    wl.one_stream = args.one_stream
    log(f"inputs resident: {torch.cuda.memory_allocated() / 2**30:.2f} GiB")
    res = wl.measure(args.steps, args.warmup, serial=not args.no_serial)
    ms_per_step = res["ms_per_step"]
    log(f"timed {args.steps} steps: {ms_per_step:.3f} ms/step")
    dominant = next(iter(res["kernels"]))
    roofline = roofline_of(res["kernels"], dominant, load_traffic(name, K, fused is not None), K)
    roofline["copy_kernel_GBps"] = copy_GBps
    roofline["atomic_adds_Gps"] = atomic_Gups      # what bounds scan_edges: one such add per scanned edge
    roofline["random_lookups_Gps"] = lookup_Gps    # 8-byte reads of random table entries: the adjacency pass does one per scanned edge
    roofline["gather_256B_rows_GBps"] = gather_GBps  # csgs_gather_rows on 1 Mi random rows of 256 bytes (read + write)
    roofline["mfma_f64_loop_TFLOPs"] = mfma_TF[False]       # the GEMM's instruction back to back, operands in registers
    roofline["mfma_f64_lds_loop_TFLOPs"] = mfma_TF[True]    # the GEMM's inner loop without global loads and barriers
    if "scan_edges" in res["kernels"]:
        per_launch = res["per_step"]["edges_scanned"] / res["kernels"]["scan_edges"]["launches_per_step"]
        roofline["scan_edges_adds_Gps"] = per_launch / (res["kernels"]["scan_edges"]["avg_us"] * 1e-6) / 1e9

    # the other way through a layer (one kernel instead of two, or two instead of one): the same schedule, timed the same
    # way on its own buffers, so that the two stand beside each other in every line
    other = None
    if not args.no_layer_compare:
        alt = "h" if fused is None else None
        wo = mk(cfg, 48 + args.warmup, K, fused=alt)
        wo.one_stream = args.one_stream
        ro = wo.measure(48, args.warmup, serial=False)
        pick = ("layer_forward",) if alt else ("aggregate", "layer_gemm")
        other = dict(layer_compute="csgs_layer_forward (Z stays in LDS)" if alt else "csgs_aggregate + csgs_layer_gemm",
                     steps=48, ms_per_step=ro["ms_per_step"],
                     kernels={k: {a: round(b, 3) for a, b in ro["kernels"][k].items()} for k in pick if k in ro["kernels"]})
        log(f"layer compute the other way ({other['layer_compute']}): {ro['ms_per_step']:.3f} ms/step over 48 steps; " +
            ", ".join(f"{k} {v['avg_us']:.1f} us per launch" for k, v in other["kernels"].items()))
        del wo, ro

    cpu_baseline = None
    if not args.no_cpu_baseline:
        import chain
        n_cpu = N_CPU
        # the oracle is single-threaded: keep it on one core for the leg (restored afterwards)
        pinned = None
        try:
            allowed = sorted(os.sched_getaffinity(0))
            pinned = allowed[len(allowed) // 2]
            os.sched_setaffinity(0, {pinned})
        except (AttributeError, OSError):
            allowed = None
        t0 = time.perf_counter()
        cpu_nnz = 0
        for it in range(args.warmup, args.warmup + n_cpu):
            osteps = chain.oracle_chain(g, X, wl.Ws, wl.batches[it], cfg.skew, wl.B, wl.seed, it, bf16)
            cpu_nnz += sum(o.sm.adj_nnz for o in osteps)
            if it == res["sizes_it"]:   # spot check: the GPU step of the same batch (the first of the first full group) drew the same nodes
                for l, o in enumerate(osteps):
                    got = res["sizes"][l]
                    assert got["n_next"] == o.sm.n_next and got["nnz"] == o.sm.adj_nnz and got["remote"] == o.rc.remote_total
        cpu_s = time.perf_counter() - t0
        if pinned is not None:
            os.sched_setaffinity(0, set(allowed))
        cpu_baseline = dict(value=cpu_nnz / cpu_s, unit="sampled edges/s", cores=1, kind="oracle",
                            sample=f"{n_cpu} whole steps of the same workload ({cpu_s:.1f} s)",
                            ms_per_step=cpu_s / n_cpu * 1e3, nproc=os.cpu_count(), cpu_model=cpu_model(),
                            pinned_to_core=pinned)
        log(f"oracle on 1 core: {cpu_s / n_cpu * 1e3:.0f} ms/step")

    t1 = None
    if not args.no_theorem1:
        t1 = wl.theorem1_sweep()
        log("Theorem-1 skew, D = 4, 8, 16, 32: remote nodes of the bottom layer " +
            ", ".join(f"{x['bottom_layer_remote_nodes']} (expected {x['bottom_layer_expected_remote_nodes']:.1f}, s = {x['layers'][-1]['skew']:g})" for x in t1))

    backward = None
    if not args.no_backward:
        backward = wl.measure_backward(args.steps)
        log(f"backward pass alone: {backward['ms_per_step']:.3f} ms/step, gradient GEMMs {backward['gemm_TFLOPs']:.1f} TFLOP/s")

    sweep = None
    if args.sweep_instances:
        sweep = []
        for Ks in [int(x) for x in args.sweep_instances.split(",") if x]:
            n_st = (48 + Ks - 1) // Ks * Ks
            n_wu = (8 + Ks - 1) // Ks * Ks
            ws_ = mk(cfg, n_st + n_wu, Ks)
            rk = ws_.measure(n_st, n_wu, serial=False)
            se = rk["kernels"]["scan_edges"]
            sweep.append(dict(instances=Ks, ms_per_step=rk["ms_per_step"], scan_edges_us_per_launch=se["avg_us"],
                              scan_edges_alg_GBps=se.get("alg_GBps"),
                              scan_edges_adds_Gps=rk["per_step"]["edges_scanned"] / se["launches_per_step"] / (se["avg_us"] * 1e-6) / 1e9,
                              kernels_us_per_launch={k: round(v["avg_us"], 2) for k, v in rk["kernels"].items()}))
            log(f"{Ks} instances per call: {rk['ms_per_step']:.3f} ms/step, scan_edges {se['avg_us']:.1f} us per launch")
            del ws_
            torch.cuda.empty_cache()

    scaled = None
    if not args.no_scaled and args.scale == 1:
        del wl
        torch.cuda.empty_cache()
        sc = 16
        cfg_s = dataclasses.replace(cfg, batch=cfg.batch * sc, samples=cfg.samples * sc)
        rs = mk(cfg_s, 8, 1).measure(6, 2)
        tr = load_traffic(f"{cfg.name}_x{sc}", 1)
        shown = ("aggregate", "layer_gemm", "layer_forward", "scan_edges", "adj_fused", "cand_emit")
        scaled = dict(workload=f"{cfg.name} x{sc}: batch {cfg_s.batch}, {cfg_s.samples} samples/layer",
                      ms_per_step=rs["ms_per_step"], one_stream_ms_per_step=rs["serial_ms_per_step"],
                      sampled_edges_per_s=rs["per_step"]["sampled_edges"] / (rs["ms_per_step"] * 1e-3),
                      per_step=rs["per_step"], aggregate_GBps=rs["aggregate_GBps"], gemm_TFLOPs=rs["gemm_TFLOPs"],
                      rooflines=[roofline_of(rs["kernels"], k, tr, 1) for k in rs["kernels"] if k in shown],
                      kernels={k: {a: round(b, 3) for a, b in v.items()} for k, v in rs["kernels"].items()})
        fmt = lambda v, f: "-" if v is None else format(v, f)
        log(f"scaled x{sc}: {rs['ms_per_step']:.3f} ms/step, aggregate {fmt(rs['aggregate_GBps'], '.0f')} GB/s, "
            f"gemm {fmt(rs['gemm_TFLOPs'], '.1f')} TFLOP/s" +
            (f", layer_forward {rs['kernels']['layer_forward']['TFLOPs']:.1f} TFLOP/s" if "layer_forward" in rs["kernels"] else ""))

    dims = synth.layer_dims(cfg)
    out = dict(
        metric="sampled-aggregation HBM GB/s + sampled edges/s per GCN layer; step time",
        value=res["per_step"]["sampled_edges"] / (ms_per_step * 1e-3), unit="sampled edges/s",
        n_gpus=1, steps=args.steps, warmup=args.warmup, ms_per_step=ms_per_step, higher_is_better=True,
        scaling="weak", vs_baseline=None,
        dtype="f64", data="synthetic",     # sums and products in double (vector ALU, fp64 matrix cores); weights and CDF in u64
        config=dict(workload=f"{name}: N={g.n_nodes}, nnz={g.nnz}, {cfg.n_parts} partitions, batch {cfg.batch}, "
                             f"{cfg.samples} samples/layer, {len(dims)} layers {dims}, skew {cfg.skew}",
                    precision=("bf16 features, " if bf16 else "f32 features, ") + "u64 fixed-point weights and CDF, f64 accumulation, f32 outputs",
                    per_step=res["per_step"]),
        one_stream_ms_per_step=res["serial_ms_per_step"],
        mini_batches_per_call=K, smaller_first_group=res["smaller_group"],
        schedule=(f"{K} consecutive mini-batches per library call, sampling then compute of every group in order on one stream; each part "
                  if args.one_stream else
                  f"{K} consecutive mini-batches per sampling call, such groups round-robin on {args.samplers} streams (own "
                  "workspace each), layer compute of all batches " + ("of a group in the same launches" if not args.no_batch_compute and K > 1
                                                                      else "in order") + " on one more stream; each part ") +
                 ("replayed from a HIP graph" if res["graphs"] else "launched call by call"),
        aggregate_GBps=res["aggregate_GBps"], gemm_TFLOPs=res["gemm_TFLOPs"],
        scanned_edges_per_s=res["per_step"]["edges_scanned"] / (ms_per_step * 1e-3),
        layer_compute="csgs_aggregate + csgs_layer_gemm" if fused is None else f"csgs_layer_forward ({fused})", layer_compute_other=other,
        roofline=roofline, cpu_baseline=cpu_baseline, backward=backward, theorem1_sweep=t1, instances_sweep=sweep,
        kernels={k: {a: round(b, 3) for a, b in v.items()} for k, v in res["kernels"].items()}, scaled=scaled)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
