"""Runs one sampled mini-batch through the CPU oracle and through the HIP library on the
same seeded inputs and compares every output.  Used by the GPU parity tests and the smoke check."""
from __future__ import annotations

from types import SimpleNamespace

import numpy as np

import oracle
from paper_2101_07706_amd import synth

RTOL, ATOL = 1e-4, 1e-5          # fp32 aggregation and GEMM outputs (stated target of the build)
P_RTOL = 2.5e-7                  # p_incl, adj_val: fp64 results rounded to fp32, libm differences <= 2 ulp


def oracle_chain(g, X, Ws, S0, skew, B, seed, it, bf16=False, auto_D=None):
    """Top-down sampling then bottom-up compute.  Ws: bottom layer first.  Returns per-step records.
    skew = inf: "Local" version.  auto_D: skew by Theorem 1 with this constant, `skew` its upper bound."""
    M = len(Ws)
    steps = []
    S = np.ascontiguousarray(S0, np.int32)
    for l in range(M):
        pr = oracle.build_probs(g, S, skew, auto=None if auto_D is None else (auto_D, B))
        sm = oracle.sample_layer(g, S, pr, B, seed, it, l)
        rc = oracle.remote_count(sm.S_next, g.local_lo, g.local_hi, g.part_bounds)
        steps.append(SimpleNamespace(S=S, pr=pr, sm=sm, rc=rc))
        S = sm.S_next
    Xs = synth.to_bf16_bits(X) if bf16 else X
    H = None
    for l in range(M - 1, -1, -1):
        st = steps[l]
        W = Ws[M - 1 - l]
        if l == M - 1:
            X_local = Xs[g.local_lo:g.local_hi]
            X_remote = Xs[st.rc.remote_ids]
            st.Z = oracle.aggregate(st.sm.adj_rowptr, st.sm.adj_col, st.sm.adj_val, X_local, X_remote, st.rc.src_row)
        else:
            st.Z = oracle.aggregate(st.sm.adj_rowptr, st.sm.adj_col, st.sm.adj_val, H, relu_on_input=True)
        st.H = oracle.layer_gemm(st.Z, W)
        H = st.H
    return steps


def gpu_chain(g, X, Ws, S0, skew, B, seed, it, bf16=False, dg=None, adj_cap=None, auto_D=None, device_counts=False,
              chained=False):
    if device_counts or chained:
        return gpu_chain_device_counts(g, X, Ws, S0, skew, B, seed, it, bf16, dg, adj_cap, auto_D, chained)
    import torch
    from paper_2101_07706_amd import pipeline
    dev = torch.device("cuda:0")
    dg = dg or pipeline.DeviceGraph(g, dev)
    M = len(Ws)
    nS_max = max(len(S0), B)
    ws = pipeline.Workspace(g.n_nodes, nS_max, B, g.nnz, dev)
    if bf16:
        Xd = torch.from_numpy(synth.to_bf16_bits(X).view(np.int16)).to(dev)
    else:
        Xd = torch.from_numpy(X).to(dev)
    Wd = [torch.from_numpy(W).to(dev) for W in Ws]
    steps = []
    S = torch.from_numpy(np.ascontiguousarray(S0, np.int32)).to(dev)
    for l in range(M):
        Sh = S.cpu().numpy().astype(np.int64)
        cap = adj_cap or int((g.rowptr[Sh + 1] - g.rowptr[Sh]).sum())
        lb = pipeline.LayerBuffers(S.numel(), B, g.n_nodes, cap, dg.n_parts, dev)
        pipeline.sample_step(dg, ws, S, skew, B, seed, it, l, lb, auto_D=auto_D)
        n = int(lb.n_next.item())
        steps.append(SimpleNamespace(S=S, lb=lb, n_next=n, status=int(lb.status.item())))
        S = lb.S_next[:n].clone()
    H = None
    for l in range(M - 1, -1, -1):
        st = steps[l]
        lb = st.lb
        nS = st.S.numel()
        W = Wd[M - 1 - l]
        Z = torch.full((nS, W.shape[0]), float("nan"), dtype=torch.float32, device=dev)
        Hn = torch.full((nS, W.shape[1]), float("nan"), dtype=torch.float32, device=dev)
        if l == M - 1:
            r = int(lb.remote_total.item())
            X_local = Xd[g.local_lo:g.local_hi]
            X_remote = Xd[lb.remote_ids[:r].long()]      # stands in for the exchange of remote rows
            args = (lb, nS, X_local, X_remote, True, False, W)
        else:
            args = (lb, nS, H, None, False, True, W)
        pipeline.compute_step(*args, Z, Hn)
        st.Z, st.H = Z, Hn
        # the same layer through the one-kernel call, on the same inputs: once with Z asked for, once without
        Zf, Hf, Hf2 = torch.full_like(Z, float("nan")), torch.full_like(Hn, float("nan")), torch.full_like(Hn, float("nan"))
        st.fused = pipeline.compute_step(*args, Zf, Hf, fused="hz")
        if st.fused:
            assert pipeline.compute_step(*args, None, Hf2, fused="h")
            st.Zf, st.Hf, st.Hf2 = Zf, Hf, Hf2
        H = Hn
    torch.cuda.synchronize()
    # workspace must be back in its prepared (all-zero) state
    from paper_2101_07706_amd import csgs
    clean = csgs.csgs_workspace_clean_bytes(g.n_nodes) // 8
    assert int(torch.count_nonzero(ws.buf[:clean]).item()) == 0, "workspace not restored"
    return steps, ws


def gpu_chain_device_counts(g, X, Ws, S0, skew, B, seed, it, bf16, dg, adj_cap, auto_D, chained=False):
    """The same chain enqueued without the host reading anything back in between: every layer's
    row count stays on the device (the previous layer's n_next), arrays have their capacity
    sizes, the staged remote rows come from csgs_gather_rows.  chained: layers after the first
    pass no row array at all, their rows are the set the previous csgs_sample_layer produced."""
    import torch
    from paper_2101_07706_amd import csgs, pipeline
    dev = torch.device("cuda:0")
    dg = dg or pipeline.DeviceGraph(g, dev)
    M = len(Ws)
    nS_max = max(len(S0), B)
    ws = pipeline.Workspace(g.n_nodes, nS_max, B, g.nnz, dev)
    Xd = torch.from_numpy(synth.to_bf16_bits(X).view(np.int16) if bf16 else X).to(dev)
    Wd = [torch.from_numpy(W).to(dev) for W in Ws]
    cap = adj_cap or min(g.nnz, 1 << 26)
    lbs = [pipeline.LayerBuffers(nS_max, B, g.n_nodes, cap, dg.n_parts, dev) for _ in range(M)]
    Zs = [torch.full((len(S0) if l == 0 else B, Wd[M - 1 - l].shape[0]), float("nan"), dtype=torch.float32, device=dev)
          for l in range(M)]
    Hs = [torch.full((len(S0) if l == 0 else B, Wd[M - 1 - l].shape[1]), float("nan"), dtype=torch.float32, device=dev)
          for l in range(M)]
    Zf, Hf, fused = [torch.full_like(z, float("nan")) for z in Zs], [torch.full_like(h, float("nan")) for h in Hs], [False] * M
    staged = torch.zeros((B, Xd.shape[1]), dtype=Xd.dtype, device=dev)
    S0d = torch.from_numpy(np.ascontiguousarray(S0, np.int32)).to(dev)
    torch.cuda.synchronize()
    # ---- nothing below reads device memory on the host until the final synchronize
    for l in range(M):
        S = S0d if l == 0 else (None if chained else lbs[l - 1].S_next)
        nS_dev = None if (l == 0 or chained) else lbs[l - 1].n_next
        pipeline.sample_step(dg, ws, S, skew, B, seed, it, l, lbs[l], auto_D=auto_D, nS_dev=nS_dev)
    pipeline.stage_remote_rows(lbs[M - 1], Xd, staged)
    X_local = Xd[g.local_lo:g.local_hi]
    for l in range(M - 1, -1, -1):
        nS = len(S0) if l == 0 else B
        nS_dev = None if l == 0 else lbs[l - 1].n_next
        if l == M - 1:
            args = (lbs[l], nS, X_local, staged, True, False, Wd[0])
        else:
            args = (lbs[l], nS, Hs[l + 1], None, False, True, Wd[M - 1 - l])
        pipeline.compute_step(*args, Zs[l], Hs[l], nS_dev=nS_dev)
        fused[l] = pipeline.compute_step(*args, Zf[l], Hf[l], nS_dev=nS_dev, fused="hz")
    torch.cuda.synchronize()
    steps = []
    for l in range(M):
        n_rows = len(S0) if l == 0 else int(lbs[l - 1].n_next.item())
        S = S0d if l == 0 else lbs[l - 1].S_next[:n_rows]
        # rows past the device count must be untouched
        assert bool(torch.isnan(Zs[l][n_rows:]).all()) and bool(torch.isnan(Hs[l][n_rows:]).all()), f"layer {l}: wrote past the row count"
        steps.append(SimpleNamespace(S=S, lb=lbs[l], n_next=int(lbs[l].n_next.item()), status=int(lbs[l].status.item()),
                                     Z=Zs[l][:n_rows], H=Hs[l][:n_rows], fused=fused[l]))
        if fused[l]:
            assert bool(torch.isnan(Zf[l][n_rows:]).all()) and bool(torch.isnan(Hf[l][n_rows:]).all()), f"layer {l}: the one-kernel call wrote past the row count"
            steps[-1].Zf, steps[-1].Hf = Zf[l][:n_rows], Hf[l][:n_rows]
    clean = csgs.csgs_workspace_clean_bytes(g.n_nodes) // 8
    assert int(torch.count_nonzero(ws.buf[:clean]).item()) == 0, "workspace not restored"
    return steps, ws


def gpu_chain_instances(g, X, Ws, S0s, skew, B, seed, it, bf16, auto_D=None, chained=True, batched_compute=False):
    """len(S0s) mini-batches sampled by the same library calls (instance k: rows S0s[k], iteration
    it + k), then the layer compute of every instance -- instance by instance, or, with
    batched_compute, all instances in the same launches (the _n forms).  Returns one list of steps
    per instance."""
    import torch
    from paper_2101_07706_amd import pipeline
    dev = torch.device("cuda:0")
    dg = pipeline.DeviceGraph(g, dev)
    M, K, n0 = len(Ws), len(S0s), len(S0s[0])
    assert all(len(s) == n0 for s in S0s)
    nS_max = max(n0, B)
    cap = min(g.nnz, 1 << 24)
    lbs = [pipeline.LayerBuffers(nS_max, B, g.n_nodes, cap, dg.n_parts, dev, n_inst=K) for _ in range(M)]
    ws = pipeline.Workspace(g.n_nodes, nS_max, B, g.nnz, dev, n_inst=K, inst_stride=lbs[0].stride)
    Xd = torch.from_numpy(synth.to_bf16_bits(X).view(np.int16) if bf16 else X).to(dev)
    Wd = [torch.from_numpy(W).to(dev) for W in Ws]
    for k in range(K):
        lbs[0].inst(k).S0[:n0].copy_(torch.from_numpy(np.ascontiguousarray(S0s[k], np.int32)))
    torch.cuda.synchronize()
    for l in range(M):
        if l == 0:
            S, nS_dev = lbs[0].S0[:n0], None
        elif chained:
            S, nS_dev = None, None
        else:
            S, nS_dev = lbs[l - 1].S_next, lbs[l - 1].n_next
        pipeline.sample_step(dg, ws, S, skew, B, seed, it, l, lbs[l], auto_D=auto_D, nS_dev=nS_dev)
    X_local = Xd[g.local_lo:g.local_hi]
    if batched_compute:
        return _instances_batched_compute(g, lbs, ws, Xd, X_local, Wd, n0, B, K, dev)
    staged = torch.zeros((B, Xd.shape[1]), dtype=Xd.dtype, device=dev)
    out = []
    for k in range(K):
        lk = [lb.inst(k) for lb in lbs]
        Zs = [torch.full((n0 if l == 0 else B, Wd[M - 1 - l].shape[0]), float("nan"), dtype=torch.float32, device=dev)
              for l in range(M)]
        Hs = [torch.full((n0 if l == 0 else B, Wd[M - 1 - l].shape[1]), float("nan"), dtype=torch.float32, device=dev)
              for l in range(M)]
        pipeline.stage_remote_rows(lk[M - 1], Xd, staged)
        for l in range(M - 1, -1, -1):
            nS = n0 if l == 0 else B
            nS_dev = None if l == 0 else lk[l - 1].n_next
            if l == M - 1:
                pipeline.compute_step(lk[l], nS, X_local, staged, True, False, Wd[0], Zs[l], Hs[l], nS_dev=nS_dev)
            else:
                pipeline.compute_step(lk[l], nS, Hs[l + 1], None, False, True, Wd[M - 1 - l], Zs[l], Hs[l], nS_dev=nS_dev)
        torch.cuda.synchronize()
        steps = []
        for l in range(M):
            n_rows = n0 if l == 0 else int(lk[l - 1].n_next.item())
            steps.append(SimpleNamespace(S=None, lb=lk[l], n_next=int(lk[l].n_next.item()), status=int(lk[l].status.item()),
                                         Z=Zs[l][:n_rows], H=Hs[l][:n_rows]))
        out.append(steps)
    clean = csgs_clean_words(g.n_nodes)
    per = ws.bytes_per_inst // 8
    for k in range(K):
        assert int(torch.count_nonzero(ws.buf[k * per:k * per + clean]).item()) == 0, f"workspace {k} not restored"
    return out


def _instances_batched_compute(g, lbs, ws, Xd, X_local, Wd, n0, B, K, dev):
    import torch
    from paper_2101_07706_amd import pipeline
    M = len(Wd)
    rows = [n0 if l == 0 else B for l in range(M)]
    Zs = [torch.full((K, rows[l], Wd[M - 1 - l].shape[0]), float("nan"), dtype=torch.float32, device=dev) for l in range(M)]
    Hs = [torch.full((K, rows[l], Wd[M - 1 - l].shape[1]), float("nan"), dtype=torch.float32, device=dev) for l in range(M)]
    staged = torch.zeros((K, B, Xd.shape[1]), dtype=Xd.dtype, device=dev)
    nbytes = lambda t: t.stride(0) * t.element_size()
    pipeline.stage_remote_rows(lbs[M - 1], Xd, staged[0], out_stride=nbytes(staged))
    for l in range(M - 1, -1, -1):
        nS_dev = None if l == 0 else lbs[l - 1].n_next
        if l == M - 1:
            pipeline.compute_step(lbs[l], rows[l], X_local, staged[0], True, False, Wd[0], Zs[l][0], Hs[l][0], nS_dev=nS_dev,
                                  strides=(0, nbytes(staged), nbytes(Zs[l]), nbytes(Hs[l])))
        else:
            pipeline.compute_step(lbs[l], rows[l], Hs[l + 1][0], None, False, True, Wd[M - 1 - l], Zs[l][0], Hs[l][0], nS_dev=nS_dev,
                                  strides=(nbytes(Hs[l + 1]), 0, nbytes(Zs[l]), nbytes(Hs[l])))
    torch.cuda.synchronize()
    out = []
    for k in range(K):
        lk = [lb.inst(k) for lb in lbs]
        steps = []
        for l in range(M):
            n_rows = n0 if l == 0 else int(lk[l - 1].n_next.item())
            assert bool(torch.isnan(Zs[l][k, n_rows:]).all()) and bool(torch.isnan(Hs[l][k, n_rows:]).all()), \
                f"instance {k} layer {l}: wrote past the row count"
            steps.append(SimpleNamespace(S=None, lb=lk[l], n_next=int(lk[l].n_next.item()), status=int(lk[l].status.item()),
                                         Z=Zs[l][k, :n_rows], H=Hs[l][k, :n_rows]))
        out.append(steps)
    return out


def csgs_clean_words(n_nodes):
    from paper_2101_07706_amd import csgs
    return csgs.csgs_workspace_clean_bytes(n_nodes) // 8


def u64(t):
    return t.cpu().numpy().view(np.uint64)


def assert_close(got, want, rtol, atol, what):
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    assert got.shape == want.shape, what
    err = np.abs(got - want)
    tol = atol + rtol * np.abs(want)
    bad = ~(err <= tol)    # a NaN on either side is outside every tolerance
    if bad.any():
        i = np.unravel_index(np.argmax(np.where(np.isnan(err), np.inf, err - tol)), err.shape)
        raise AssertionError(f"{what}: {int(bad.sum())} of {bad.size} outside tolerance; worst at {i}: "
                             f"got {got[i]!r} want {want[i]!r} err {err[i]:.3e} tol {tol[i]:.3e}")
    return float((err / tol).max()) if err.size else 0.0


# (layer, elements of Z, elements of H that differ in any bit between csgs_layer_forward and the two calls, size of Z)
# of the layers compare_chain() has seen, for the tests' logs
fused_bit_differences = []


def compare_chain(osteps, gsteps, check_compute=True):
    worst = {}
    for l, (o, gs) in enumerate(zip(osteps, gsteps)):
        lb = gs.lb
        assert gs.status == 0, f"layer {l}: status {gs.status}"
        st = lb.stats_host()
        pr, sm, rc = o.pr, o.sm, o.rc
        for k in ("n_cand", "n_local", "n_remote", "edges_scanned", "w_local", "w_remote", "total", "shift", "skew_fx"):
            assert int(getattr(st, k)) == int(getattr(pr, k)), f"layer {l}: stats.{k}"
        n = pr.n_cand
        np.testing.assert_array_equal(lb.cand_id[:n].cpu().numpy(), pr.cand_id, err_msg=f"layer {l} cand_id")
        np.testing.assert_array_equal(u64(lb.cand_w[:n]), pr.cand_w, err_msg=f"layer {l} cand_w")
        np.testing.assert_array_equal(u64(lb.cdf[:n]), pr.cdf, err_msg=f"layer {l} cdf")
        qg = lb.q[:n].cpu().numpy()
        np.testing.assert_array_equal(qg, pr.q, err_msg=f"layer {l} q")
        # sort order of the probabilities: keys (weight desc, id asc) are integers, so exact
        wsk_g = np.diff(np.concatenate([[np.uint64(0)], u64(lb.cdf[:n])]))
        wsk_o = np.diff(np.concatenate([[np.uint64(0)], pr.cdf]))
        np.testing.assert_array_equal(np.lexsort((pr.cand_id, -wsk_g.astype(np.int64))),
                                      np.lexsort((pr.cand_id, -wsk_o.astype(np.int64))))
        m = sm.n_next
        assert gs.n_next == m, f"layer {l}: n_next {gs.n_next} != {m}"
        np.testing.assert_array_equal(lb.S_next[:m].cpu().numpy(), sm.S_next, err_msg=f"layer {l} S_next")
        np.testing.assert_array_equal(lb.mult[:m].cpu().numpy(), sm.mult, err_msg=f"layer {l} mult")
        assert_close(lb.p_incl[:m].cpu().numpy(), sm.p_incl, P_RTOL, 0.0, f"layer {l} p_incl")
        nS = len(o.S)
        np.testing.assert_array_equal(lb.adj_rowptr[:nS + 1].cpu().numpy(), sm.adj_rowptr, err_msg=f"layer {l} adj_rowptr")
        nnz = sm.adj_nnz
        assert int(lb.adj_nnz.item()) == nnz
        np.testing.assert_array_equal(lb.adj_col[:nnz].cpu().numpy(), sm.adj_col, err_msg=f"layer {l} adj_col")
        assert_close(lb.adj_val[:nnz].cpu().numpy(), sm.adj_val, P_RTOL, 0.0, f"layer {l} adj_val")
        assert int(lb.remote_total.item()) == rc.remote_total, f"layer {l} remote_total"
        np.testing.assert_array_equal(lb.per_part.cpu().numpy(), rc.per_part, err_msg=f"layer {l} per_part")
        np.testing.assert_array_equal(lb.src_row[:m].cpu().numpy(), rc.src_row, err_msg=f"layer {l} src_row")
        np.testing.assert_array_equal(lb.remote_ids[:rc.remote_total].cpu().numpy(), rc.remote_ids)
        if check_compute:
            worst[f"Z{l}"] = assert_close(gs.Z.cpu().numpy(), o.Z, RTOL, ATOL, f"layer {l} Z")
            worst[f"H{l}"] = assert_close(gs.H.cpu().numpy(), o.H, RTOL, ATOL, f"layer {l} H")
            if getattr(gs, "fused", False):   # csgs_layer_forward ran on the same inputs as the two calls
                worst[f"Zf{l}"] = assert_close(gs.Zf.cpu().numpy(), o.Z, RTOL, ATOL, f"layer {l} Z of the one-kernel call")
                worst[f"Hf{l}"] = assert_close(gs.Hf.cpu().numpy(), o.H, RTOL, ATOL, f"layer {l} H of the one-kernel call")
                if hasattr(gs, "Hf2"):
                    assert bool((gs.Hf2 == gs.Hf).all()), f"layer {l}: H depends on whether Z is asked for"
                # the two paths round Z at the same point; they differ in the order of the double sums of a row
                fused_bit_differences.append((l, int((gs.Zf != gs.Z).sum().item()), int((gs.Hf != gs.H).sum().item()), gs.Zf.numel()))
    return worst


def config_inputs(name, it=0):
    cfg = synth.CONFIGS[name]
    g = synth.make_graph(cfg)
    X = synth.make_features(cfg.n_nodes, cfg.feat_dim, cfg.seed)
    Ws = [synth.glorot_uniform(fi, fo, cfg.seed) for fi, fo in synth.layer_dims(cfg)]
    S0 = synth.make_batch(g, cfg.batch, cfg.seed, it)
    return cfg, g, X, Ws, S0
