"""HIP library against the CPU oracle, element by element, through the C-ABI binding.
Integer outputs (candidates, fixed-point weights, CDF, sampled ids, multiplicities, adjacency
structure, remote counts) must be bit-exact; fp32 aggregation and GEMM within 1e-4 rel + 1e-5 abs."""
import sys

import numpy as np
import pytest

import chain
import oracle
from paper_2101_07706_amd import synth

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def dev():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2101_07706_amd import csgs
    csgs.lib()
    return torch.device("cuda:0")


def run_config(name, it=0, skew=None, bf16=None):
    cfg, g, X, Ws, S0 = chain.config_inputs(name, it)
    skew = cfg.skew if skew is None else skew
    bf16 = (cfg.feat_dtype == "bf16") if bf16 is None else bf16
    say(f"[{name}] it={it} skew={skew} bf16={bf16} nnz={g.nnz}")
    osteps = chain.oracle_chain(g, X, Ws, S0, skew, cfg.samples, 1234 + cfg.seed, it, bf16)
    gsteps, _ = chain.gpu_chain(g, X, Ws, S0, skew, cfg.samples, 1234 + cfg.seed, it, bf16)
    del chain.fused_bit_differences[:]
    worst = chain.compare_chain(osteps, gsteps)
    say(f"[{name}] layers: " + ", ".join(
        f"nS={len(o.S)} E={o.pr.edges_scanned} nc={o.pr.n_cand} n'={o.sm.n_next} nnz={o.sm.adj_nnz} rem={o.rc.remote_total}"
        for o in osteps) + f" worst err/tol {worst}")
    say(f"[{name}] one-kernel layer call against the two calls, (layer, Z elements, H elements that differ, of): {chain.fused_bit_differences}")


def test_tiny_config(dev):
    run_config("tiny")
    run_config("tiny", it=3, skew=1.0)


def test_medium_config(dev):
    run_config("medium")


def test_mid_config(dev):
    run_config("mid")


_cache = {}


def cached_inputs(name):
    """Full-size inputs are generated once per test session."""
    if name not in _cache:
        _cache.clear()          # one big graph in host memory at a time
        _cache[name] = chain.config_inputs(name)
    return _cache[name]


def run_full_size(name, skews, its=(0,)):
    from paper_2101_07706_amd import pipeline
    cfg, g, X, Ws, _ = cached_inputs(name)
    bf16 = cfg.feat_dtype == "bf16"
    dg = pipeline.DeviceGraph(g, torch.device("cuda:0"))
    for skew in skews:
        for it in its:
            S0 = synth.make_batch(g, cfg.batch, cfg.seed, it)
            say(f"[{name}] full size, skew={skew} it={it}")
            osteps = chain.oracle_chain(g, X, Ws, S0, skew, cfg.samples, 1234 + cfg.seed, it, bf16)
            gsteps, _ = chain.gpu_chain(g, X, Ws, S0, skew, cfg.samples, 1234 + cfg.seed, it, bf16, dg=dg)
            worst = chain.compare_chain(osteps, gsteps)
            say(f"[{name}] " + ", ".join(
                f"nS={len(o.S)} E={o.pr.edges_scanned} nc={o.pr.n_cand} n'={o.sm.n_next} nnz={o.sm.adj_nnz} rem={o.rc.remote_total}"
                for o in osteps) + f" worst err/tol {max(worst.values()):.3f}")
    return osteps


def run_instances(name, K, chained, batched):
    """K mini-batches of consecutive iterations through the same sampling calls (n_inst = K in the
    workspace descriptor) and, with `batched`, through the same compute launches (the _n forms):
    every instance equals the oracle's chain for its batch and iteration."""
    it = 4
    if name in ("large", "dense"):
        cfg, g, X, Ws, _ = cached_inputs(name)
    else:
        cfg, g, X, Ws, _ = chain.config_inputs(name, it)
    S0s = [synth.make_batch(g, cfg.batch, cfg.seed, it + k) for k in range(K)]
    bf16 = cfg.feat_dtype == "bf16"
    say(f"[{name}] {K} instances per call, chained={chained}, compute batched={batched}")
    auto_D = 8.0 if (name == "tiny" and not chained) else None
    got = chain.gpu_chain_instances(g, X, Ws, S0s, cfg.skew, cfg.samples, 1234 + cfg.seed, it, bf16, auto_D=auto_D,
                                    chained=chained, batched_compute=batched)
    for k in range(K):
        osteps = chain.oracle_chain(g, X, Ws, S0s[k], cfg.skew, cfg.samples, 1234 + cfg.seed, it + k, bf16, auto_D=auto_D)
        worst = chain.compare_chain(osteps, got[k])
        say(f"[{name}] instance {k}: n' {[o.sm.n_next for o in osteps]} worst err/tol {max(worst.values()):.3f}")


def test_dense_config_skew_sweep(dev, monkeypatch):
    """Dense-neighborhood config at full size (114 M edges), every output element by element, over
    the skew sweep; the bottom layer's remote count must fall as the skew grows.  Once more with the
    weight scan forced through owner blocks (left to itself the library scans these sizes with atomics)."""
    from paper_2101_07706_amd import pipeline
    cfg = synth.CONFIGS["dense"]
    remote = []
    for s in cfg.skews:
        osteps = run_full_size("dense", [s])
        remote.append(osteps[-1].rc.remote_total)
    say(f"[dense] remote nodes of the bottom layer over skews {cfg.skews}: {remote}")
    assert remote[0] > remote[-1]
    monkeypatch.setattr(pipeline, "DEFAULT_SCAN_MODE", 2)
    run_full_size("dense", [cfg.skews[len(cfg.skews) // 2]])


def test_dense_config_instances(dev):
    """Dense-neighborhood config, 8 mini-batches per sampling call and per compute launch (the form bench.py times)."""
    run_instances("dense", 8, True, True)


def test_large_config(dev):
    """Large config at full size (the workload bench.py times), bf16 features, two different batches."""
    run_full_size("large", [synth.CONFIGS["large"].skew], its=(0, 7))


def test_large_config_scaled(dev):
    """Large config with batch and samples per layer times 16 (the scaled-up variant bench.py also times):
    every output element by element."""
    from paper_2101_07706_amd import pipeline
    cfg, g, X, Ws, _ = cached_inputs("large")
    sc = 16
    dg = pipeline.DeviceGraph(g, torch.device("cuda:0"))
    S0 = synth.make_batch(g, cfg.batch * sc, cfg.seed, 0)
    say(f"[large x{sc}] batch {len(S0)}, {cfg.samples * sc} samples per layer")
    osteps = chain.oracle_chain(g, X, Ws, S0, cfg.skew, cfg.samples * sc, 1234 + cfg.seed, 0, True)
    gsteps, _ = chain.gpu_chain(g, X, Ws, S0, cfg.skew, cfg.samples * sc, 1234 + cfg.seed, 0, True, dg=dg)
    worst = chain.compare_chain(osteps, gsteps)
    say(f"[large x{sc}] " + ", ".join(f"nS={len(o.S)} E={o.pr.edges_scanned} n'={o.sm.n_next} nnz={o.sm.adj_nnz}" for o in osteps)
        + f" worst err/tol {max(worst.values()):.3f}")


class SmallGraph:
    """Random symmetric-normalised graph with self-loops and a few isolated (self-loop only) nodes."""

    def __init__(self, n, avg_deg, seed, lo, hi, n_parts=3):
        rng = np.random.default_rng(seed)
        m = int(n * avg_deg / 2)
        u = rng.integers(0, n, m)
        v = rng.integers(0, n, m)
        keep = u != v
        u, v = u[keep], v[keep]
        keys = np.unique(np.concatenate([u * n + v, v * n + u, np.arange(n) * (n + 1)]))
        row, col = keys // n, keys % n
        deg = np.bincount(row, minlength=n)
        self.n_nodes = n
        self.rowptr = np.zeros(n + 1, np.int64)
        np.cumsum(deg, out=self.rowptr[1:])
        self.colidx = col.astype(np.int32)
        self.val = (1.0 / np.sqrt(deg[row].astype(np.float64) * deg[col])).astype(np.float32)
        self.local_lo, self.local_hi = lo, hi
        self.rownorm2_max = 1.0
        self.part_bounds = np.array(sorted({0, lo, hi, n}), np.int32)

    @property
    def nnz(self):
        return len(self.colidx)


@pytest.mark.parametrize("n,avg_deg,nS,B,skew,lo,hi", [
    (1, 0, 1, 1, 1.0, 0, 1),            # a single self-loop
    (70, 3, 1, 5, 2.0, 10, 40),         # one row
    (70, 3, 70, 500, 16.0, 0, 70),      # everything local, B far above the candidate count
    (1000, 8, 65, 64, 4.0, 300, 600),   # ragged: one row more than a wavefront multiple
    (5000, 40, 333, 257, 8.0, 0, 1250),
    (5000, 2, 1023, 1025, 2.5, 4000, 5000),
    (3000, 5, 17, 4100, 1.0, 1000, 1000),   # empty local range: every candidate is remote
])
def test_small_graphs(dev, n, avg_deg, nS, B, skew, lo, hi):
    g = SmallGraph(n, avg_deg, seed=n + nS, lo=lo, hi=hi)
    rng = np.random.default_rng(7)
    S0 = rng.choice(n, size=nS, replace=False).astype(np.int32)       # unsorted on purpose
    F = 12
    X = rng.standard_normal((n, F)).astype(np.float32)
    Ws = [synth.glorot_uniform(F, 9, 1), synth.glorot_uniform(9, 6, 2)]
    say(f"[small] n={n} nS={nS} B={B} skew={skew}")
    osteps = chain.oracle_chain(g, X, Ws, S0, skew, B, 42, 7)
    gsteps, _ = chain.gpu_chain(g, X, Ws, S0, skew, B, 42, 7)
    chain.compare_chain(osteps, gsteps)


# ---------------------------------------------------------------- weight scan through owner blocks
@pytest.fixture
def owner_scan(monkeypatch):
    """Workspaces made during the test ask for the owner-block form of the weight scan whatever the size
    (left to itself the library takes it only for launches of a million edges or more)."""
    from paper_2101_07706_amd import pipeline
    monkeypatch.setattr(pipeline, "DEFAULT_SCAN_MODE", 2)


@pytest.mark.parametrize("n,avg_deg,nS,B,skew,lo,hi", [
    (1, 0, 1, 1, 1.0, 0, 1), (70, 3, 1, 5, 2.0, 10, 40), (70, 3, 70, 500, 16.0, 0, 70), (1000, 8, 65, 64, 4.0, 300, 600),
    (5000, 40, 333, 257, 8.0, 0, 1250), (5000, 2, 1023, 1025, 2.5, 4000, 5000), (3000, 5, 17, 4100, 1.0, 1000, 1000),
    (9000, 30, 2000, 700, 4.0, 100, 8900),     # several owner blocks, the last one partly outside the range
])
def test_small_graphs_owner_scan(dev, owner_scan, n, avg_deg, nS, B, skew, lo, hi):
    test_small_graphs(dev, n, avg_deg, nS, B, skew, lo, hi)


@pytest.mark.parametrize("name", ["tiny", "medium", "mid"])
def test_configs_owner_scan(dev, owner_scan, name):
    run_config(name)
    run_config_device_counts(name, it=2)


def test_weight_scan_modes_agree_and_bad_mode_is_rejected(dev):
    """The same call with scan_mode 1 (atomics) and 2 (owner blocks) writes identical candidates, weights and CDF."""
    from paper_2101_07706_amd import csgs, pipeline
    cfg, g, X, Ws, S0 = chain.config_inputs("medium", 3)
    dg = pipeline.DeviceGraph(g, dev)
    S0d = torch.from_numpy(np.ascontiguousarray(S0, np.int32)).to(dev)
    outs = []
    for mode in (1, 2):
        ws = pipeline.Workspace(g.n_nodes, len(S0), cfg.samples, g.nnz, dev, scan_mode=mode)
        lb = pipeline.LayerBuffers(len(S0), cfg.samples, g.n_nodes, 1, dg.n_parts, dev)
        csgs.csgs_build_probs(dg.c, S0d, cfg.skew, lb.cand_id, lb.cand_w, lb.cdf, lb.q, lb.stats, ws.desc, lb.status)
        torch.cuda.synchronize()
        assert int(lb.status.item()) == 0
        outs.append(lb)
    n = int(outs[0].stats_host().n_cand)
    assert n == int(outs[1].stats_host().n_cand) and n > 0
    for f in ("cand_id", "cand_w", "cdf", "q", "stats"):
        a, b = getattr(outs[0], f), getattr(outs[1], f)
        assert torch.equal(a[:n] if f != "stats" else a, b[:n] if f != "stats" else b), f
    bad = pipeline.Workspace(g.n_nodes, len(S0), cfg.samples, g.nnz, dev, scan_mode=3)
    with pytest.raises(csgs.CsgsError):
        csgs.csgs_build_probs(dg.c, S0d, cfg.skew, outs[0].cand_id, outs[0].cand_w, outs[0].cdf, None, outs[0].stats, bad.desc,
                              outs[0].status)


@pytest.mark.parametrize("policy", ["auto_D4", "auto_D32", "auto_D0", "local"])
@pytest.mark.parametrize("n,avg_deg,nS,B,lo,hi", [(1000, 8, 65, 64, 300, 600), (5000, 40, 333, 257, 0, 1250),
                                                  (3000, 5, 17, 4100, 1000, 1000), (70, 3, 70, 500, 0, 70)])
def test_skew_policies(dev, policy, n, avg_deg, nS, B, lo, hi):
    """Skew chosen on the device by Theorem 1 (Eq. 12), and the Local version, against the oracle."""
    g = SmallGraph(n, avg_deg, seed=n + nS, lo=lo, hi=hi)
    rng = np.random.default_rng(11)
    S0 = rng.choice(n, size=nS, replace=False).astype(np.int32)
    X = rng.standard_normal((n, 12)).astype(np.float32)
    Ws = [synth.glorot_uniform(12, 9, 1), synth.glorot_uniform(9, 6, 2)]
    if policy == "local":
        kw = dict(skew=float("inf"))
    else:
        kw = dict(skew=1024.0, auto_D=float(policy[6:]))
    say(f"[policy] {policy} n={n} nS={nS} B={B}")
    if policy == "local" and lo == hi:
        with pytest.raises(oracle.OracleError):      # no local candidate at all: nothing can be drawn
            chain.oracle_chain(g, X, Ws, S0, B=B, seed=42, it=7, **kw)
        return
    osteps = chain.oracle_chain(g, X, Ws, S0, B=B, seed=42, it=7, **kw)
    gsteps, _ = chain.gpu_chain(g, X, Ws, S0, B=B, seed=42, it=7, **kw)
    chain.compare_chain(osteps, gsteps)
    say(f"[policy] skew_fx per layer: {[o.pr.skew_fx for o in osteps]} remote: {[o.rc.remote_total for o in osteps]}")


def test_tiny_config_theorem1_sweep(dev):
    """The paper's sweep of D (Section 5.2: 4, 8, 16, 32) on the Tiny configuration."""
    cfg, g, X, Ws, S0 = chain.config_inputs("tiny")
    remote = []
    for D in (4.0, 8.0, 16.0, 32.0):
        osteps = chain.oracle_chain(g, X, Ws, S0, 4096.0, cfg.samples, 77, 0, auto_D=D)
        gsteps, _ = chain.gpu_chain(g, X, Ws, S0, 4096.0, cfg.samples, 77, 0, auto_D=D)
        chain.compare_chain(osteps, gsteps)
        remote.append(sum(o.rc.remote_total for o in osteps))
        say(f"[tiny] D={D}: skew_fx {[o.pr.skew_fx for o in osteps]} remote {remote[-1]}")
    assert remote[-1] < remote[0]


def test_dense_config_theorem1_sweep(dev):
    """The paper's sweep of D (Section 5.2: 4, 8, 16, 32) on the Dense-neighbourhood configuration at full
    size, the skew chosen on the device from the candidate counts of each layer (Theorem 1, Eq. 12).  Every
    output element by element; the bottom layer's sampled remote nodes (what the method reduces) fall as D
    grows and agree with their expectation sum_{j in R} p_j (Eq. 4 with Eq. 8) within sampling noise."""
    from paper_2101_07706_amd import pipeline
    cfg, g, X, Ws, _ = cached_inputs("dense")
    dg = pipeline.DeviceGraph(g, torch.device("cuda:0"))
    S0 = synth.make_batch(g, cfg.batch, cfg.seed, 0)
    B = cfg.samples
    remote, expect, skews = [], [], []
    for D in (4.0, 8.0, 16.0, 32.0):
        say(f"[dense] Theorem-1 skew, D={D}")
        osteps = chain.oracle_chain(g, X, Ws, S0, 4096.0, B, 1234 + cfg.seed, 0, auto_D=D)
        gsteps, _ = chain.gpu_chain(g, X, Ws, S0, 4096.0, B, 1234 + cfg.seed, 0, dg=dg, auto_D=D)
        chain.compare_chain(osteps, gsteps)
        bottom = osteps[-1]
        pr = bottom.pr
        q = np.diff(np.concatenate([[0], pr.cdf.astype(np.float64)])) / float(pr.total)
        is_remote = (pr.cand_id < g.local_lo) | (pr.cand_id >= g.local_hi)
        p = 1.0 - (1.0 - q[is_remote]) ** B
        mean, sd = float(p.sum()), float(np.sqrt((p * (1 - p)).sum()))     # the draws' inclusion indicators are negatively correlated: sd is an upper bound
        remote.append(bottom.rc.remote_total)
        expect.append(mean)
        skews.append([o.pr.skew_fx / 16 for o in osteps])
        assert int(gsteps[-1].lb.remote_total.item()) == bottom.rc.remote_total
        assert abs(bottom.rc.remote_total - mean) <= 5 * sd + 1, (D, bottom.rc.remote_total, mean, sd)
    say(f"[dense] D = 4, 8, 16, 32: skew per layer {skews}; remote nodes of the bottom layer {remote}, expected {[round(e, 1) for e in expect]}")
    assert remote[0] > remote[-1] and all(a >= b for a, b in zip(expect, expect[1:]))


def _subgraph_variant(dev, g, X, W, skew, B, seed):
    """Subgraph sampler of Section 5.1: candidates = all (training) nodes, one draw of the subgraph's
    node set from the skewed distribution, sampled adjacency restricted to the drawn nodes, one
    full convolution on it.  Returns nothing; asserts parity of every output."""
    from paper_2101_07706_amd import csgs, pipeline
    n = g.n_nodes
    rows_all = np.arange(n, dtype=np.int32)
    pr = oracle.build_probs(g, rows_all, skew)
    dr = oracle.draw_nodes(pr, B, seed, 0, 0)
    adj = oracle.sampled_adjacency(g, dr.S_next, dr)
    rc = oracle.remote_count(dr.S_next, g.local_lo, g.local_hi, g.part_bounds)
    Z = oracle.aggregate(adj.adj_rowptr, adj.adj_col, adj.adj_val, X[g.local_lo:g.local_hi], X[rc.remote_ids], rc.src_row)
    H = oracle.layer_gemm(Z, W)

    dg = pipeline.DeviceGraph(g, dev)
    ws = pipeline.Workspace(n, n, B, g.nnz, dev)
    lb = pipeline.LayerBuffers(n, B, n, int(g.nnz), dg.n_parts, dev)
    Sd = torch.from_numpy(rows_all).to(dev)
    csgs.csgs_build_probs(dg.c, Sd, skew, lb.cand_id, lb.cand_w, lb.cdf, lb.q, lb.stats, ws.desc, lb.status)
    csgs.csgs_draw_nodes(n, lb.cand_id, lb.cdf, lb.stats, B, seed, 0, 0, lb.S_next, lb.mult, lb.p_incl, lb.n_next,
                         ws.desc, lb.status)
    m = int(lb.n_next.item())
    assert m == dr.n_next
    np.testing.assert_array_equal(lb.S_next[:m].cpu().numpy(), dr.S_next)
    np.testing.assert_array_equal(lb.mult[:m].cpu().numpy(), dr.mult)
    np.testing.assert_array_equal(chain.u64(lb.cdf[:pr.n_cand]), pr.cdf)
    rows = lb.S_next[:m].clone()
    csgs.csgs_sampled_adjacency(dg.c, rows, lb.adj_rowptr[:m + 1], lb.adj_col, lb.adj_val, lb.adj_nnz, ws.desc, lb.status)
    csgs.csgs_remote_count(lb.S_next, lb.n_next, g.local_lo, g.local_hi, dg.part_bounds, lb.remote_total, lb.per_part,
                           lb.src_row, lb.remote_ids)
    torch.cuda.synchronize()
    assert int(lb.status.item()) == 0
    assert int(lb.adj_nnz.item()) == adj.adj_nnz
    np.testing.assert_array_equal(lb.adj_rowptr[:m + 1].cpu().numpy(), adj.adj_rowptr)
    np.testing.assert_array_equal(lb.adj_col[:adj.adj_nnz].cpu().numpy(), adj.adj_col)
    chain.assert_close(lb.adj_val[:adj.adj_nnz].cpu().numpy(), adj.adj_val, chain.P_RTOL, 0.0, "subgraph adj_val")
    r = int(lb.remote_total.item())
    assert r == rc.remote_total
    Xd = torch.from_numpy(X).to(dev)
    Zd = torch.full((m, X.shape[1]), float("nan"), dtype=torch.float32, device=dev)
    Hd = torch.full((m, W.shape[1]), float("nan"), dtype=torch.float32, device=dev)
    pipeline.compute_step(lb, m, Xd[g.local_lo:g.local_hi], Xd[lb.remote_ids[:r].long()], True, False,
                          torch.from_numpy(W).to(dev), Zd, Hd)
    torch.cuda.synchronize()
    chain.assert_close(Zd.cpu().numpy(), Z, chain.RTOL, chain.ATOL, "subgraph Z")
    chain.assert_close(Hd.cpu().numpy(), H, chain.RTOL, chain.ATOL, "subgraph H")
    say(f"[subgraph] n={n} nodes drawn {m} of {B}, edges {adj.adj_nnz}, remote {r}")


def test_subgraph_sampler_small(dev):
    g = SmallGraph(3000, 12, seed=5, lo=500, hi=1500)
    rng = np.random.default_rng(0)
    X = rng.standard_normal((3000, 16)).astype(np.float32)
    _subgraph_variant(dev, g, X, synth.glorot_uniform(16, 8, 3), 4.0, 450, 99)


def test_subgraph_sampler_medium_graph(dev):
    """All 262,144 nodes of the Medium graph as candidates, subgraph of 4500 draws (the size the paper uses)."""
    cfg, g, X, Ws, _ = cached_inputs("medium")
    _subgraph_variant(dev, g, X, Ws[0], cfg.skew, 4500, 7)


def _drop_rows(g, rows):
    """Remove every edge of the given rows (they become empty rows; P is no longer symmetric, which
    the method does not need)."""
    keep = np.ones(g.nnz, bool)
    for i in rows:
        keep[g.rowptr[i]:g.rowptr[i + 1]] = False
    row = np.repeat(np.arange(g.n_nodes), np.diff(g.rowptr))[keep]
    g.colidx, g.val = g.colidx[keep], g.val[keep]
    g.rowptr = np.zeros(g.n_nodes + 1, np.int64)
    np.cumsum(np.bincount(row, minlength=g.n_nodes), out=g.rowptr[1:])


@pytest.mark.parametrize("case", ["scattered", "leading_trailing", "long_run"])
def test_empty_rows_in_S(dev, case):
    n = 6000
    g = SmallGraph(n, 30, seed=11, lo=1000, hi=3000)
    rng = np.random.default_rng(3)
    if case == "scattered":
        empty = rng.choice(n, size=n // 2, replace=False)
        S0 = rng.choice(n, size=700, replace=False)
    elif case == "leading_trailing":
        S0 = rng.choice(n, size=300, replace=False)
        empty = np.concatenate([S0[:40], S0[-25:], S0[100:103]])
    else:   # more consecutive empty rows than one staged slice can hold, then ordinary rows
        S0 = rng.permutation(n)[:4000]
        empty = S0[200:3500]
    _drop_rows(g, empty)
    X = rng.standard_normal((n, 8)).astype(np.float32)
    Ws = [synth.glorot_uniform(8, 8, 1), synth.glorot_uniform(8, 4, 2)]
    say(f"[empty rows] {case}: nnz={g.nnz}")
    osteps = chain.oracle_chain(g, X, Ws, S0.astype(np.int32), 4.0, 300, 5, 1)
    gsteps, _ = chain.gpu_chain(g, X, Ws, S0.astype(np.int32), 4.0, 300, 5, 1)
    chain.compare_chain(osteps, gsteps)


def test_status_bits_and_restored_workspace(dev):
    from paper_2101_07706_amd import csgs, pipeline
    g = SmallGraph(500, 6, seed=1, lo=0, hi=200)
    S = torch.from_numpy(np.arange(0, 100, dtype=np.int32)).to(dev)
    B = 64
    ws = pipeline.Workspace(g.n_nodes, 128, B, g.nnz, dev)
    clean = csgs.csgs_workspace_clean_bytes(g.n_nodes) // 8

    def fresh(cand_cap, adj_cap):
        return pipeline.LayerBuffers(128, B, cand_cap, adj_cap, len(g.part_bounds) - 1, dev)

    # candidate capacity too small
    dg = pipeline.DeviceGraph(g, dev)
    lb = fresh(10, 4096)
    pipeline.sample_step(dg, ws, S, 2.0, B, 1, 0, 0, lb)
    torch.cuda.synchronize()
    assert int(lb.status.item()) & csgs.ST_CAND_OVERFLOW
    assert lb.stats_host().n_cand == oracle.build_probs(g, S.cpu().numpy(), 2.0).n_cand
    assert int(torch.count_nonzero(ws.buf[:clean]).item()) == 0
    # adjacency capacity too small
    lb = fresh(g.n_nodes, 3)
    pipeline.sample_step(dg, ws, S, 2.0, B, 1, 0, 0, lb)
    torch.cuda.synchronize()
    assert int(lb.status.item()) == csgs.ST_ADJ_OVERFLOW
    assert int(lb.adj_nnz.item()) > 3
    assert int(torch.count_nonzero(ws.buf[:clean]).item()) == 0
    # a NaN edge value and an id outside the graph
    g2 = SmallGraph(500, 6, seed=1, lo=0, hi=200)
    g2.val = g2.val.copy()
    g2.val[g2.rowptr[5]] = np.nan
    dg2 = pipeline.DeviceGraph(g2, dev)
    lb = fresh(g.n_nodes, 4096)
    S_bad = S.clone()
    S_bad[7] = 100000
    pipeline.sample_step(dg2, ws, S_bad, 2.0, B, 1, 0, 0, lb)
    torch.cuda.synchronize()
    st = int(lb.status.item())
    assert st & csgs.ST_BAD_EDGE_VALUE and st & csgs.ST_BAD_NODE_ID
    assert int(torch.count_nonzero(ws.buf[:clean]).item()) == 0
    # rows without any edge: no candidates
    g3 = SmallGraph(50, 0, seed=2, lo=0, hi=25)
    g3.rowptr = np.zeros(51, np.int64)
    g3.colidx = np.zeros(1, np.int32)
    g3.val = np.zeros(1, np.float32)
    dg3 = pipeline.DeviceGraph(g3, dev)
    ws3 = pipeline.Workspace(50, 128, B, 64, dev)
    lb = fresh(50, 16)
    pipeline.sample_step(dg3, ws3, S[:10].contiguous(), 2.0, B, 1, 0, 0, lb)
    torch.cuda.synchronize()
    assert int(lb.status.item()) & csgs.ST_EMPTY_CANDIDATES
    assert int(lb.n_next.item()) == 0 and int(lb.adj_nnz.item()) == 0 and int(lb.remote_total.item()) == 0
    # after all that the same workspace still gives exact results
    lb = fresh(g.n_nodes, 4096)
    pipeline.sample_step(dg, ws, S, 2.0, B, 1, 0, 0, lb)
    torch.cuda.synchronize()
    pr = oracle.build_probs(g, S.cpu().numpy(), 2.0)
    sm = oracle.sample_layer(g, S.cpu().numpy(), pr, B, 1, 0, 0)
    assert int(lb.status.item()) == 0
    np.testing.assert_array_equal(lb.S_next[:sm.n_next].cpu().numpy(), sm.S_next)
    np.testing.assert_array_equal(chain.u64(lb.cdf[:pr.n_cand]), pr.cdf)


def _random_adj(rng, n_rows, n_cols, max_len):
    lens = rng.integers(0, max_len + 1, n_rows)
    lens[rng.integers(0, n_rows)] = 0
    lens = np.minimum(lens, n_cols)
    rowptr = np.zeros(n_rows + 1, np.int32)
    np.cumsum(lens, out=rowptr[1:])
    col = np.concatenate([np.sort(rng.choice(n_cols, size=l, replace=False)) for l in lens] + [np.zeros(0, np.int64)])
    val = (rng.standard_normal(len(col)) * 3).astype(np.float32)
    return rowptr, col.astype(np.int32), val


@pytest.mark.parametrize("F,bf16", [(64, False), (128, False), (256, False), (512, False), (300, False),
                                    (602, False), (7, False), (100, True), (100, False), (33, True), (256, True)])
@pytest.mark.parametrize("mode", ["compact_relu", "src_row"])
def test_aggregate_shapes(dev, F, bf16, mode):
    from paper_2101_07706_amd import csgs
    rng = np.random.default_rng(F)
    n_rows, n_cols = 777, 500
    rowptr, col, val = _random_adj(rng, n_rows, n_cols, 150)
    say(f"[aggregate] F={F} bf16={bf16} mode={mode} nnz={len(col)}")
    Xl = rng.standard_normal((n_cols if mode == "compact_relu" else 900, F)).astype(np.float32)
    Xr = rng.standard_normal((60, F)).astype(np.float32)
    if bf16:
        Xl_h, Xr_h = synth.to_bf16_bits(Xl), synth.to_bf16_bits(Xr)
        Xl_d = torch.from_numpy(Xl_h.view(np.int16)).to(dev)
        Xr_d = torch.from_numpy(Xr_h.view(np.int16)).to(dev)
    else:
        Xl_h, Xr_h = Xl, Xr
        Xl_d, Xr_d = torch.from_numpy(Xl).to(dev), torch.from_numpy(Xr).to(dev)
    t = lambda a: torch.from_numpy(a).to(dev)
    n_next = torch.tensor([n_cols], dtype=torch.int32, device=dev)
    Z = torch.full((n_rows, F), float("nan"), dtype=torch.float32, device=dev)
    if mode == "compact_relu":
        want = oracle.aggregate(rowptr, col, val, Xl_h, relu_on_input=True)
        csgs.csgs_aggregate(t(rowptr), t(col), t(val), n_next, Xl_d, None, None, True, Z)
    else:
        src = np.where(rng.random(n_cols) < 0.8, rng.integers(0, 900, n_cols), -1 - rng.integers(0, 60, n_cols)).astype(np.int32)
        want = oracle.aggregate(rowptr, col, val, Xl_h, Xr_h, src)
        csgs.csgs_aggregate(t(rowptr), t(col), t(val), n_next, Xl_d, Xr_d, t(src), False, Z)
    torch.cuda.synchronize()
    chain.assert_close(Z.cpu().numpy(), want, chain.RTOL, chain.ATOL, f"aggregate F={F}")


@pytest.mark.parametrize("F,bf16", [(256, False), (100, True), (512, False), (47, False)])
def test_aggregate_hub_rows_and_edges_that_do_not_count(dev, F, bf16):
    """Rows of a few hundred to a few thousand kept edges beside short and empty ones (the block-wide path for the
    longest, sums carried from one round of staged edges into the next for the others), at the widths of the
    configurations; and edges whose column or source row lies outside the tables: they contribute nothing, also
    when the row they would have read holds NaN."""
    from paper_2101_07706_amd import csgs
    rng = np.random.default_rng(7 * F)
    n_rows, n_cols, n_loc, n_rem = 700, 4000, 5000, 300
    lens = rng.poisson(3, n_rows)
    lens[rng.choice(n_rows, 12, replace=False)] = rng.integers(200, 3000, 12)
    lens[[0, 63, 64, 699]] = [257, 256, 0, 1000]
    rowptr = np.zeros(n_rows + 1, np.int32)
    np.cumsum(lens, out=rowptr[1:])
    col = np.concatenate([np.sort(rng.choice(n_cols, size=l, replace=False)) for l in lens]).astype(np.int32)
    val = rng.standard_normal(len(col)).astype(np.float32)
    src = np.where(rng.random(n_cols) < 0.85, rng.integers(1, n_loc, n_cols), -1 - rng.integers(0, n_rem, n_cols)).astype(np.int32)
    Xl = rng.standard_normal((n_loc, F)).astype(np.float32)
    Xr = rng.standard_normal((n_rem, F)).astype(np.float32)
    Xl[0] = np.nan          # row 0 of the local table: what a dropped edge's load may touch; no valid edge points at it
    if bf16:
        Xl_h, Xr_h = synth.to_bf16_bits(Xl), synth.to_bf16_bits(Xr)
        Xl_d, Xr_d = torch.from_numpy(Xl_h.view(np.int16)).to(dev), torch.from_numpy(Xr_h.view(np.int16)).to(dev)
    else:
        Xl_h, Xr_h = Xl, Xr
        Xl_d, Xr_d = torch.from_numpy(Xl).to(dev), torch.from_numpy(Xr).to(dev)
    want = oracle.aggregate(rowptr, col, val, Xl_h, Xr_h, src)
    # the same operator with edges that must be dropped spliced in: columns beyond the column count, negative columns,
    # columns whose source row is outside either table
    bad_src = src.copy()
    bad_cols = rng.choice(n_cols, 40, replace=False)
    keep = ~np.isin(col, bad_cols)
    want_bad = oracle.aggregate(np.concatenate([[0], np.cumsum(np.add.reduceat(keep, rowptr[:-1]) * (lens > 0))]).astype(np.int32),
                                col[keep], val[keep], Xl_h, Xr_h, src)
    bad_src[bad_cols[:20]] = n_loc + 5            # beyond the local table
    bad_src[bad_cols[20:]] = -1 - (n_rem + 3)     # beyond the staged remote rows
    col2 = col.copy()
    t = lambda a: torch.from_numpy(a).to(dev)
    n_next = torch.tensor([n_cols], dtype=torch.int32, device=dev)
    say(f"[aggregate] hubs: F={F} bf16={bf16} nnz={len(col)} longest rows {np.sort(lens)[-4:]}")
    Z = torch.full((n_rows, F), float("nan"), dtype=torch.float32, device=dev)
    csgs.csgs_aggregate(t(rowptr), t(col), t(val), n_next, Xl_d, Xr_d, t(src), False, Z)
    torch.cuda.synchronize()
    chain.assert_close(Z.cpu().numpy(), want, chain.RTOL, chain.ATOL, f"aggregate with hub rows F={F}")
    Z.fill_(float("nan"))
    csgs.csgs_aggregate(t(rowptr), t(col2), t(val), n_next, Xl_d, Xr_d, t(bad_src), False, Z)
    torch.cuda.synchronize()
    chain.assert_close(Z.cpu().numpy(), want_bad, chain.RTOL, chain.ATOL, f"source rows outside the tables F={F}")
    # columns at or beyond the column count, and negative ones
    n_small = torch.tensor([n_cols - 500], dtype=torch.int32, device=dev)
    keep = col < n_cols - 500
    want_cut = oracle.aggregate(np.concatenate([[0], np.cumsum(np.add.reduceat(keep, rowptr[:-1]) * (lens > 0))]).astype(np.int32),
                                col[keep], val[keep], Xl_h, Xr_h, src)
    Z.fill_(float("nan"))
    csgs.csgs_aggregate(t(rowptr), t(col), t(val), n_small, Xl_d, Xr_d, t(src), False, Z)
    torch.cuda.synchronize()
    chain.assert_close(Z.cpu().numpy(), want_cut, chain.RTOL, chain.ATOL, f"columns beyond the column count F={F}")
    # no table at all: every row is a zero row
    Z.fill_(float("nan"))
    csgs.csgs_aggregate(t(rowptr), t(col), t(val), n_next, Xl_d[:0], None, t(src), False, Z)
    torch.cuda.synchronize()
    assert bool((Z == 0).all())


@pytest.mark.parametrize("K,N,bf16", [(256, 256, False), (100, 256, True), (256, 47, False), (64, 64, False), (128, 256, False),
                                      (256, 41, True), (33, 5, False), (7, 100, True), (252, 300, False), (1, 1, False)])
@pytest.mark.parametrize("mode", ["compact_relu", "src_row"])
def test_layer_forward_shapes(dev, K, N, bf16, mode):
    """csgs_layer_forward against the oracle's aggregation followed by its layer product: hub rows (block-wide path,
    sums carried over rounds of staged edges), empty rows, edges that do not count, a row count that is not a multiple
    of a block's 32 rows, a device row count below the capacity, Z asked for or not, widths with ragged K chunks and
    ragged column tiles."""
    from paper_2101_07706_amd import csgs
    rng = np.random.default_rng(1000 * K + N)
    n_rows, n_cols, n_loc, n_rem = 717, 3000, 3500, 200
    lens = rng.poisson(3, n_rows)
    lens[rng.choice(n_rows, 10, replace=False)] = rng.integers(60, 1500, 10)
    lens[[0, 31, 32, 63, 716]] = [257, 256, 0, 65, 700]
    rowptr = np.zeros(n_rows + 1, np.int32)
    np.cumsum(lens, out=rowptr[1:])
    col = np.concatenate([np.sort(rng.choice(n_cols, size=l, replace=False)) for l in lens]).astype(np.int32)
    val = rng.standard_normal(len(col)).astype(np.float32)
    compact = mode == "compact_relu"
    Xl = rng.standard_normal((n_cols if compact else n_loc, K)).astype(np.float32)
    Xr = rng.standard_normal((n_rem, K)).astype(np.float32)
    src = np.where(rng.random(n_cols) < 0.85, rng.integers(1, n_loc, n_cols), -1 - rng.integers(0, n_rem, n_cols)).astype(np.int32)
    bad = rng.choice(n_cols, 30, replace=False)       # columns whose source row lies outside the tables
    src[bad[:15]] = n_loc + 7
    src[bad[15:]] = -1 - (n_rem + 2)
    W = (rng.standard_normal((K, N)) / np.sqrt(K)).astype(np.float32)
    if bf16:
        Xl_h, Xr_h = synth.to_bf16_bits(Xl), synth.to_bf16_bits(Xr)
        Xl_d, Xr_d = torch.from_numpy(Xl_h.view(np.int16)).to(dev), torch.from_numpy(Xr_h.view(np.int16)).to(dev)
    else:
        Xl_h, Xr_h = Xl, Xr
        Xl_d, Xr_d = torch.from_numpy(Xl).to(dev), torch.from_numpy(Xr).to(dev)
    t = lambda a: torch.from_numpy(a).to(dev)
    n_small = n_cols - 300                              # columns at or beyond the column count do not count either
    n_next = torch.tensor([n_small], dtype=torch.int32, device=dev)
    keep = col < n_small
    if not compact:
        keep &= ~np.isin(col, bad)
    rp_keep = np.concatenate([[0], np.cumsum(np.add.reduceat(keep, rowptr[:-1]) * (lens > 0))]).astype(np.int32)
    if compact:
        Z_want = oracle.aggregate(rp_keep, col[keep], val[keep], Xl_h, relu_on_input=True)
        call = lambda Z, H, nS_dev=None: csgs.csgs_layer_forward(t(rowptr), t(col), t(val), n_next, Xl_d, None, None, True, Wd, H, Z, nS_dev=nS_dev)
        two = lambda Z: csgs.csgs_aggregate(t(rowptr), t(col), t(val), n_next, Xl_d, None, None, True, Z)
    else:
        Z_want = oracle.aggregate(rp_keep, col[keep], val[keep], Xl_h, Xr_h, src)
        call = lambda Z, H, nS_dev=None: csgs.csgs_layer_forward(t(rowptr), t(col), t(val), n_next, Xl_d, Xr_d, t(src), False, Wd, H, Z, nS_dev=nS_dev)
        two = lambda Z: csgs.csgs_aggregate(t(rowptr), t(col), t(val), n_next, Xl_d, Xr_d, t(src), False, Z)
    H_want = oracle.layer_gemm(Z_want, W)
    Wd = t(W)
    assert csgs.csgs_layer_forward_supported(Xl_d, None if compact else Xr_d)
    say(f"[layer_forward] K={K} N={N} bf16={bf16} mode={mode} nnz={len(col)} longest rows {np.sort(lens)[-3:]}")
    nan = lambda *shape: torch.full(shape, float("nan"), dtype=torch.float32, device=dev)
    Z, H, H2 = nan(n_rows, K), nan(n_rows, N), nan(n_rows, N)
    call(Z, H)
    call(None, H2)
    torch.cuda.synchronize()
    chain.assert_close(Z.cpu().numpy(), Z_want, chain.RTOL, chain.ATOL, f"Z of the one-kernel call K={K}")
    worst = chain.assert_close(H.cpu().numpy(), H_want, chain.RTOL, chain.ATOL, f"H of the one-kernel call K={K} N={N}")
    assert bool((H == H2).all()), "H depends on whether Z is asked for"
    # the product's input is the Z the call reports: the oracle's product of exactly that Z
    chain.assert_close(H.cpu().numpy(), oracle.layer_gemm(Z.cpu().numpy(), W), chain.RTOL, chain.ATOL, "H against the product of the reported Z")
    Z2 = nan(n_rows, K)
    two(Z2)
    torch.cuda.synchronize()
    say(f"[layer_forward] worst err/tol {worst:.3f}; elements of Z that differ in any bit from csgs_aggregate: {int((Z2 != Z).sum().item())} of {Z.numel()}")
    # a device row count below the capacity: rows past it stay untouched
    for count in (0, 1, 33, 500):
        Z, H = nan(n_rows, K), nan(n_rows, N)
        call(Z, H, nS_dev=torch.tensor([count], dtype=torch.int32, device=dev))
        torch.cuda.synchronize()
        assert bool(torch.isnan(Z[count:]).all()) and bool(torch.isnan(H[count:]).all()), f"count {count}: wrote past the row count"
        chain.assert_close(H[:count].cpu().numpy(), H_want[:count], chain.RTOL, chain.ATOL, f"device row count {count}")
        chain.assert_close(Z[:count].cpu().numpy(), Z_want[:count], chain.RTOL, chain.ATOL, f"device row count {count}, Z")


def test_layer_forward_random_shapes(dev):
    """Forty seeded random shapes (widths the call takes, any number of columns and rows, leading dimensions wider than
    the rows) against the oracle: ragged K chunks, ragged and single column tiles, blocks with fewer than 32 rows."""
    from paper_2101_07706_amd import csgs
    rng = np.random.default_rng(20240607)
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    done = 0
    while done < 40:
        K = int(rng.integers(1, 257))
        v = 1 if K <= 64 else (2 if K <= 128 else 4)
        if K % v:
            K += v - K % v
        N, n_rows, n_cols = int(rng.integers(1, 330)), int(rng.integers(1, 200)), int(rng.integers(1, 300))
        bf16 = bool(rng.integers(0, 2))
        rowptr, col, val = _random_adj(rng, n_rows, n_cols, int(rng.integers(0, 70)))
        ld = K + v * int(rng.integers(0, 3))
        X = np.zeros((n_cols, ld), np.float32)
        X[:, :K] = rng.standard_normal((n_cols, K))
        W = np.zeros((K, N + int(rng.integers(0, 5))), np.float32)
        W[:, :N] = rng.standard_normal((K, N)) / np.sqrt(K)
        relu = bool(rng.integers(0, 2))
        if bf16:
            Xh = synth.to_bf16_bits(X)
            Xd = torch.from_numpy(Xh.view(np.int16)).to(dev)[:, :K]
            Xo = Xh[:, :K]
        else:
            Xd = t(X)[:, :K]
            Xo = X[:, :K]
        Wd = t(W)[:, :N]
        Z_want = oracle.aggregate(rowptr, col, val, np.ascontiguousarray(Xo), relu_on_input=relu)
        H_want = oracle.layer_gemm(Z_want, np.ascontiguousarray(W[:, :N]))
        say(f"[layer_forward] random shape {done}: K={K} N={N} rows={n_rows} cols={n_cols} bf16={bf16} relu={relu} ld={ld} nnz={len(col)}")
        assert csgs.csgs_layer_forward_supported(Xd)
        H = torch.full((n_rows, N + 3), float("nan"), dtype=torch.float32, device=dev)
        Z = torch.full((n_rows, K + 1), float("nan"), dtype=torch.float32, device=dev)
        csgs.csgs_layer_forward(t(rowptr), t(col), t(val), torch.tensor([n_cols], dtype=torch.int32, device=dev), Xd, None, None, relu,
                                Wd, H[:, :N], Z[:, :K])
        torch.cuda.synchronize()
        chain.assert_close(Z[:, :K].cpu().numpy(), Z_want, chain.RTOL, chain.ATOL, f"random shape {done}: Z")
        chain.assert_close(H[:, :N].cpu().numpy(), H_want, chain.RTOL, chain.ATOL, f"random shape {done}: H")
        assert bool(torch.isnan(H[:, N:]).all()) and bool(torch.isnan(Z[:, K:]).all()), "wrote beyond the row width"
        done += 1


def test_layer_forward_instances_and_unsupported_widths(dev):
    """Three instances in one launch equal three separate calls bit for bit; widths the kernel does not take are refused
    before anything is enqueued."""
    from paper_2101_07706_amd import csgs
    rng = np.random.default_rng(99)
    n_inst, n_rows, n_cols, K, N = 3, 300, 400, 128, 96
    t = lambda a: torch.from_numpy(a).to(dev)
    cap = 16384
    # the instances' adjacency arrays, counts and column bounds lie `stride` bytes apart in one buffer
    stride = (4 * (n_rows + 1) + 8 * cap + 8 + 15) // 16 * 16
    buf = torch.zeros(n_inst * stride // 4, dtype=torch.int32, device=dev)
    Xs = rng.standard_normal((n_inst, n_cols, K)).astype(np.float32)
    W = (rng.standard_normal((K, N)) / np.sqrt(K)).astype(np.float32)
    Xd, Wd = t(Xs), t(W)
    views, wants = [], []
    for k in range(n_inst):
        rowptr, col, val = _random_adj(rng, n_rows, n_cols, 40)
        assert len(col) <= cap
        base = k * stride // 4
        rp = buf[base:base + n_rows + 1]
        cl = buf[base + n_rows + 1:base + n_rows + 1 + cap]
        vl = buf[base + n_rows + 1 + cap:base + n_rows + 1 + 2 * cap].view(torch.float32)
        cnt = buf[base + n_rows + 1 + 2 * cap:base + n_rows + 2 + 2 * cap]
        nn = buf[base + n_rows + 2 + 2 * cap:base + n_rows + 3 + 2 * cap]
        rp.copy_(t(rowptr)); cl[:len(col)].copy_(t(col)); vl[:len(val)].copy_(t(val))
        cnt.fill_(n_rows - 10 * k); nn.fill_(n_cols)
        views.append((rp, cl, vl, cnt, nn))
        Zw = oracle.aggregate(rowptr, col, val, Xs[k], relu_on_input=True)
        wants.append(oracle.layer_gemm(Zw, W)[:n_rows - 10 * k])
    H = torch.full((n_inst, n_rows, N), float("nan"), dtype=torch.float32, device=dev)
    Z = torch.full((n_inst, n_rows, K), float("nan"), dtype=torch.float32, device=dev)
    rp, cl, vl, cnt, nn = views[0]
    inst = csgs.InstStrides(n_inst, 0, stride, Xd.stride(0) * 4, 0, H.stride(0) * 4)
    csgs.csgs_layer_forward(rp, cl, vl, nn, Xd[0], None, None, True, Wd, H[0], Z[0], nS_dev=cnt, inst=inst, z_stride=Z.stride(0) * 4)
    torch.cuda.synchronize()
    for k in range(n_inst):
        rp, cl, vl, cnt, nn = views[k]
        H1 = torch.full((n_rows, N), float("nan"), dtype=torch.float32, device=dev)
        Z1 = torch.full((n_rows, K), float("nan"), dtype=torch.float32, device=dev)
        csgs.csgs_layer_forward(rp, cl, vl, nn, Xd[k], None, None, True, Wd, H1, Z1, nS_dev=cnt)
        torch.cuda.synchronize()
        m = n_rows - 10 * k
        assert bool((H1[:m] == H[k, :m]).all()) and bool((Z1[:m] == Z[k, :m]).all()), f"instance {k} differs from its own call"
        assert bool(torch.isnan(H[k, m:]).all()) and bool(torch.isnan(Z[k, m:]).all())
        chain.assert_close(H[k, :m].cpu().numpy(), wants[k], chain.RTOL, chain.ATOL, f"instance {k}")
    say("[layer_forward] 3 instances in one launch equal their own calls")
    for K_bad, dt in ((300, torch.float32), (512, torch.float32), (602, torch.int16), (101, torch.float32), (130, torch.float32)):
        Xb = torch.zeros((8, K_bad), dtype=dt, device=dev)
        assert not csgs.csgs_layer_forward_supported(Xb)
        with pytest.raises(csgs.CsgsError) as e:
            csgs.csgs_layer_forward(views[0][0], views[0][1], views[0][2], views[0][4], Xb, None, None, True,
                                    torch.zeros((K_bad, 8), dtype=torch.float32, device=dev),
                                    torch.zeros((n_rows, 8), dtype=torch.float32, device=dev))
        assert e.value.code == csgs.EUNSUPPORTED, K_bad
    torch.cuda.synchronize()


@pytest.mark.parametrize("mean_len,device_count", [(2, False), (2, True), (24, False), (24, True)])
def test_aggregate_many_rows(dev, mean_len, device_count):
    """Calls with tens of thousands of rows: the kernel itself decides, by the mean number of kept edges per
    row, whether leading blocks or the owning blocks take the long rows.  Both outcomes, rows of 0 to 400 edges."""
    from paper_2101_07706_amd import csgs
    rng = np.random.default_rng(1000 + mean_len)
    n_rows, n_cols, F = 40000, 6000, 64
    lens = rng.poisson(mean_len, n_rows)
    long_ones = rng.choice(n_rows, 300, replace=False)
    lens[long_ones] = rng.integers(33, 400, 300)
    lens[rng.choice(n_rows, 50, replace=False)] = 0
    rowptr = np.zeros(n_rows + 1, np.int32)
    np.cumsum(lens, out=rowptr[1:])
    col = rng.integers(0, n_cols, int(rowptr[-1])).astype(np.int32)   # (repeated columns in a row are allowed: they add up)
    val = rng.standard_normal(len(col)).astype(np.float32)
    X = rng.standard_normal((n_cols, F)).astype(np.float32)
    m = 39001 if device_count else n_rows
    say(f"[aggregate] {n_rows} rows, mean {len(col) / n_rows:.1f} edges, device count {device_count}")
    t = lambda a: torch.from_numpy(a).to(dev)
    Z = torch.full((n_rows, F), float("nan"), dtype=torch.float32, device=dev)
    cnt = torch.tensor([m], dtype=torch.int32, device=dev) if device_count else None
    csgs.csgs_aggregate(t(rowptr), t(col), t(val), None, t(X), None, None, True, Z, nS_dev=cnt)
    torch.cuda.synchronize()
    want = oracle.aggregate(rowptr[:m + 1], col[:rowptr[m]], val[:rowptr[m]], X, relu_on_input=True)
    chain.assert_close(Z[:m].cpu().numpy(), want, chain.RTOL, chain.ATOL, "Z of a call with many rows")
    assert bool(torch.isnan(Z[m:]).all())


@pytest.mark.parametrize("M,K,N", [(1, 1, 1), (33, 17, 5), (256, 64, 64), (1024, 128, 256), (2048, 602, 256),
                                   (2048, 256, 41), (4096, 300, 512), (4096, 512, 100), (8192, 100, 256),
                                   (8192, 256, 256), (8192, 256, 47), (100, 1000, 70),
                                   # one to four k beyond whole chunks of 32: folded into the last chunk
                                   (300, 36, 70), (513, 68, 47), (1000, 33, 64), (257, 66, 33), (129, 99, 20),
                                   (4096, 132, 256), (640, 35, 300), (77, 34, 16), (128, 37, 64),
                                   # 512 and more blocks of 128 x 64: the block shape of a launch for 8 mini-batches of the
                                   # largest configuration (regular shape, with and without folded tail, ragged, narrow output)
                                   (16384, 256, 256), (16384, 100, 256), (16500, 100, 256), (16421, 250, 256),
                                   (65536, 256, 47), (65541, 256, 47), (32768, 36, 128)])
def test_layer_gemm_shapes(dev, M, K, N):
    from paper_2101_07706_amd import csgs
    rng = np.random.default_rng(M + K + N)
    say(f"[gemm] {M}x{K}x{N}")
    Z = rng.standard_normal((M, K)).astype(np.float32)
    W = synth.glorot_uniform(K, N, 5)
    want = oracle.layer_gemm(Z, W)
    H = torch.full((M, N), float("nan"), dtype=torch.float32, device=dev)
    csgs.csgs_layer_gemm(torch.from_numpy(Z).to(dev), torch.from_numpy(W).to(dev), H)
    torch.cuda.synchronize()
    chain.assert_close(H.cpu().numpy(), want, chain.RTOL, chain.ATOL, f"gemm {M}x{K}x{N}")


# ---------------------------------------------------------------- row counts that stay on the device
def run_config_device_counts(name, it=0, auto_D=None):
    cfg, g, X, Ws, S0 = chain.config_inputs(name, it)
    bf16 = cfg.feat_dtype == "bf16"
    say(f"[{name}] device-side row counts, it={it} auto_D={auto_D}")
    osteps = chain.oracle_chain(g, X, Ws, S0, cfg.skew, cfg.samples, 1234 + cfg.seed, it, bf16, auto_D=auto_D)
    gsteps, _ = chain.gpu_chain(g, X, Ws, S0, cfg.skew, cfg.samples, 1234 + cfg.seed, it, bf16, auto_D=auto_D,
                                device_counts=True)
    worst = chain.compare_chain(osteps, gsteps)
    say(f"[{name}] n' per layer {[o.sm.n_next for o in osteps]} worst err/tol {max(worst.values()):.3f}")


@pytest.mark.parametrize("name", ["tiny", "medium", "mid"])
def test_chain_without_host_reads(dev, name):
    """The whole step enqueued with every layer's row count left on the device (n_dev arguments,
    capacity-sized arrays, staged remote rows by csgs_gather_rows): same results as the oracle."""
    run_config_device_counts(name)
    if name == "tiny":
        run_config_device_counts(name, it=2, auto_D=8.0)


def test_chain_without_host_reads_large(dev):
    cfg, g, X, Ws, _ = cached_inputs("large")
    S0 = synth.make_batch(g, cfg.batch, cfg.seed, 3)
    osteps = chain.oracle_chain(g, X, Ws, S0, cfg.skew, cfg.samples, 1234 + cfg.seed, 3, True)
    gsteps, _ = chain.gpu_chain(g, X, Ws, S0, cfg.skew, cfg.samples, 1234 + cfg.seed, 3, True, device_counts=True)
    worst = chain.compare_chain(osteps, gsteps)
    say(f"[large] device-side row counts: n' {[o.sm.n_next for o in osteps]} worst err/tol {max(worst.values()):.3f}")


@pytest.mark.parametrize("name", ["tiny", "medium", "mid", "large"])
def test_chain_on_prepared_rows(dev, name):
    """Layers after the first pass no row array: csgs_build_probs(S = NULL) takes the node set the
    previous csgs_sample_layer sampled, whose offsets that call prepared.  Same results as the oracle."""
    if name in ("large", "dense"):
        cfg, g, X, Ws, _ = cached_inputs(name)
        S0 = synth.make_batch(g, cfg.batch, cfg.seed, 5)
        it = 5
    else:
        it = 1
        cfg, g, X, Ws, S0 = chain.config_inputs(name, it)
    bf16 = cfg.feat_dtype == "bf16"
    say(f"[{name}] rows prepared by the previous layer")
    for auto_D in (None, 8.0) if name == "tiny" else (None,):
        osteps = chain.oracle_chain(g, X, Ws, S0, cfg.skew, cfg.samples, 1234 + cfg.seed, it, bf16, auto_D=auto_D)
        gsteps, _ = chain.gpu_chain(g, X, Ws, S0, cfg.skew, cfg.samples, 1234 + cfg.seed, it, bf16, auto_D=auto_D,
                                    chained=True)
        worst = chain.compare_chain(osteps, gsteps)
        say(f"[{name}] n' per layer {[o.sm.n_next for o in osteps]} worst err/tol {max(worst.values()):.3f}")


# ---------------------------------------------------------------- several mini-batches per call
@pytest.mark.parametrize("name,K,chained,batched", [("tiny", 3, True, False), ("tiny", 2, False, True), ("medium", 4, True, True),
                                                     ("mid", 2, True, False), ("mid", 3, True, True), ("large", 3, True, False),
                                                     ("large", 2, True, True), ("large", 8, True, True)])
def test_instances_per_call(dev, name, K, chained, batched):
    run_instances(name, K, chained, batched)


def test_instances_are_isolated(dev):
    """A fault in one instance's input (a row id outside the graph) is reported in that instance's
    status word only; the other instances of the same calls are exact."""
    from paper_2101_07706_amd import csgs, pipeline
    cfg, g, X, Ws, _ = chain.config_inputs("tiny", 0)
    B, K, it = cfg.samples, 3, 11
    S0s = [synth.make_batch(g, cfg.batch, cfg.seed, it + k) for k in range(K)]
    n0 = len(S0s[0])
    bad = S0s[1].copy()
    bad[5] = g.n_nodes + 17
    dg = pipeline.DeviceGraph(g, dev)
    nS_max = max(n0, B)
    lb = pipeline.LayerBuffers(nS_max, B, g.n_nodes, g.nnz, dg.n_parts, dev, n_inst=K)
    ws = pipeline.Workspace(g.n_nodes, nS_max, B, g.nnz, dev, n_inst=K, inst_stride=lb.stride)
    for k, S in enumerate([S0s[0], bad, S0s[2]]):
        lb.inst(k).S0[:n0].copy_(torch.from_numpy(np.ascontiguousarray(S, np.int32)))
    pipeline.sample_step(dg, ws, lb.S0[:n0], cfg.skew, B, 1234 + cfg.seed, it, 0, lb)
    torch.cuda.synchronize()
    st = [int(lb.inst(k).status.item()) for k in range(K)]
    assert st[0] == 0 and st[2] == 0 and st[1] & csgs.ST_BAD_NODE_ID, st
    for k in (0, 2):
        pr = oracle.build_probs(g, S0s[k], cfg.skew)
        sm = oracle.sample_layer(g, S0s[k], pr, B, 1234 + cfg.seed, it + k, 0)
        lk = lb.inst(k)
        assert int(lk.n_next.item()) == sm.n_next
        np.testing.assert_array_equal(lk.S_next[:sm.n_next].cpu().numpy(), sm.S_next)
        np.testing.assert_array_equal(chain.u64(lk.cdf[:pr.n_cand]), pr.cdf)
        np.testing.assert_array_equal(lk.adj_rowptr[:n0 + 1].cpu().numpy(), sm.adj_rowptr)
    clean = chain.csgs_clean_words(g.n_nodes)
    per = ws.bytes_per_inst // 8
    for k in range(K):
        assert int(torch.count_nonzero(ws.buf[k * per:k * per + clean]).item()) == 0, f"workspace {k} not restored"


def test_prepared_rows_need_a_matching_sample_layer(dev):
    """csgs_build_probs(S = NULL) is refused on the host when no csgs_sample_layer has prepared rows,
    when nS is not that call's B, when a device count is given, and after the rows were consumed."""
    from paper_2101_07706_amd import csgs, pipeline
    cfg, g, X, Ws, S0 = chain.config_inputs("tiny", 0)
    B = cfg.samples
    dg = pipeline.DeviceGraph(g, dev)
    nS_max = max(len(S0), B)
    ws = pipeline.Workspace(g.n_nodes, nS_max, B, g.nnz, dev)
    lb0 = pipeline.LayerBuffers(nS_max, B, g.n_nodes, g.nnz, dg.n_parts, dev)
    lb1 = pipeline.LayerBuffers(nS_max, B, g.n_nodes, g.nnz, dg.n_parts, dev)
    S0d = torch.from_numpy(np.ascontiguousarray(S0, np.int32)).to(dev)

    def chained(lb, nS, nS_dev=None):
        csgs.csgs_build_probs(dg.c, None, cfg.skew, lb.cand_id, lb.cand_w, lb.cdf, None, lb.stats, ws.desc, lb.status,
                              nS_dev=nS_dev, nS=nS)

    with pytest.raises(csgs.CsgsError):
        chained(lb1, B)                                   # nothing prepared yet
    pipeline.sample_step(dg, ws, S0d, cfg.skew, B, 7, 0, 0, lb0)
    with pytest.raises(csgs.CsgsError):
        chained(lb1, B - 1)                               # not the capacity of the draw
    with pytest.raises(csgs.CsgsError):
        chained(lb1, B, nS_dev=lb0.n_next)                # the count is already known
    chained(lb1, B)                                       # accepted
    with pytest.raises(csgs.CsgsError):
        chained(lb1, B)                                   # consumed
    torch.cuda.synchronize()
    assert int(lb0.status.item()) == 0 and int(lb1.status.item()) == 0
    # the accepted call equals the explicit form
    lb2 = pipeline.LayerBuffers(nS_max, B, g.n_nodes, g.nnz, dg.n_parts, dev)
    csgs.csgs_build_probs(dg.c, lb0.S_next, cfg.skew, lb2.cand_id, lb2.cand_w, lb2.cdf, None, lb2.stats, ws.desc,
                          lb2.status, nS_dev=lb0.n_next)
    torch.cuda.synchronize()
    n = int(lb2.stats_host().n_cand)
    assert n == int(lb1.stats_host().n_cand) and n > 0
    assert torch.equal(lb1.cand_id[:n], lb2.cand_id[:n]) and torch.equal(lb1.cdf[:n], lb2.cdf[:n])


def test_device_row_count_small_and_zero(dev):
    """A device count below the capacity gives exactly the result of a call with that many rows;
    a device count of zero gives an empty candidate set (status bit) and writes nothing else."""
    from paper_2101_07706_amd import csgs, pipeline
    g = SmallGraph(2000, 10, seed=11, lo=400, hi=900)
    rng = np.random.default_rng(4)
    S_full = rng.permutation(2000)[:300].astype(np.int32)
    B = 128
    dg = pipeline.DeviceGraph(g, dev)
    ws = pipeline.Workspace(g.n_nodes, 300, B, g.nnz, dev)
    Sd = torch.from_numpy(S_full).to(dev)
    for n_rows in (300, 77, 1):
        pr = oracle.build_probs(g, S_full[:n_rows], 3.0)
        sm = oracle.sample_layer(g, S_full[:n_rows], pr, B, 5, 1, 0)
        lb = pipeline.LayerBuffers(300, B, g.n_nodes, g.nnz, dg.n_parts, dev)
        lb.adj_rowptr.fill_(-7)
        cnt = torch.tensor([n_rows], dtype=torch.int32, device=dev)
        pipeline.sample_step(dg, ws, Sd, 3.0, B, 5, 1, 0, lb, nS_dev=cnt)
        torch.cuda.synchronize()
        assert int(lb.status.item()) == 0
        st = lb.stats_host()
        assert (st.n_cand, st.total, st.shift) == (pr.n_cand, pr.total, pr.shift)
        np.testing.assert_array_equal(chain.u64(lb.cdf[:pr.n_cand]), pr.cdf)
        m = int(lb.n_next.item())
        assert m == sm.n_next
        np.testing.assert_array_equal(lb.S_next[:m].cpu().numpy(), sm.S_next)
        np.testing.assert_array_equal(lb.adj_rowptr[:n_rows + 1].cpu().numpy(), sm.adj_rowptr)
        assert bool((lb.adj_rowptr[n_rows + 1:] == -7).all()), "row pointers past the device count were written"
        np.testing.assert_array_equal(lb.adj_col[:sm.adj_nnz].cpu().numpy(), sm.adj_col)
    lb = pipeline.LayerBuffers(300, B, g.n_nodes, g.nnz, dg.n_parts, dev)
    cnt = torch.zeros(1, dtype=torch.int32, device=dev)
    csgs.csgs_build_probs(dg.c, Sd, 3.0, lb.cand_id, lb.cand_w, lb.cdf, lb.q, lb.stats, ws.desc, lb.status, nS_dev=cnt)
    torch.cuda.synchronize()
    assert int(lb.status.item()) == csgs.ST_EMPTY_CANDIDATES
    assert lb.stats_host().n_cand == 0 and lb.stats_host().edges_scanned == 0
    clean = csgs.csgs_workspace_clean_bytes(g.n_nodes) // 8
    assert int(torch.count_nonzero(ws.buf[:clean]).item()) == 0


@pytest.mark.parametrize("F,bf16,off", [(64, False, 0), (100, True, 0), (602, True, 0), (33, False, 0), (7, True, 1),
                                        (256, False, 2)])
def test_gather_rows(dev, F, bf16, off):
    """csgs_gather_rows against plain indexing, for every vector width the alignment allows."""
    from paper_2101_07706_amd import csgs
    rng = np.random.default_rng(F)
    rows, cap, n = 500, 200, 137
    ld = F + off
    if bf16:
        Xh = rng.integers(-30000, 30000, (rows, ld)).astype(np.int16)
    else:
        Xh = rng.standard_normal((rows, ld)).astype(np.float32)
    ids = rng.integers(0, rows, cap).astype(np.int32)
    ids[5], ids[6] = -1, rows      # outside the table: zero rows
    Xd = torch.from_numpy(Xh).to(dev)[:, :F]
    out = torch.full((cap, ld), 99, dtype=Xd.dtype, device=dev)[:, :F]
    csgs.csgs_gather_rows(Xd, torch.from_numpy(ids).to(dev), torch.tensor([n], dtype=torch.int64, device=dev), out)
    torch.cuda.synchronize()
    want = Xh[:, :F][np.clip(ids[:n], 0, rows - 1)].copy()
    want[5] = 0
    want[6] = 0
    got = out.cpu().numpy()
    np.testing.assert_array_equal(got[:n], want)
    assert (got[n:] == 99).all(), "rows past the device count were written"


def _gemm_device_row_count(dev, rng, M, K, N, m):
    from paper_2101_07706_amd import csgs
    Z = rng.standard_normal((M, K)).astype(np.float32)
    W = rng.standard_normal((K, N)).astype(np.float32)
    Zd, Wd = torch.from_numpy(Z).to(dev), torch.from_numpy(W).to(dev)
    Zd[m:] = float("nan")          # rows beyond the count may be read; what they hold must reach nothing
    Zd[m + 1::3] = float("inf")
    H = torch.full((M, N), float("nan"), dtype=torch.float32, device=dev)
    csgs.csgs_layer_gemm(Zd, Wd, H, M_dev=torch.tensor([m], dtype=torch.int32, device=dev))
    torch.cuda.synchronize()
    chain.assert_close(H[:m].cpu().numpy(), oracle.layer_gemm(Z[:m], W), chain.RTOL, chain.ATOL, f"H with M_dev {M}x{K}x{N}")
    assert bool(torch.isnan(H[m:]).all())


def test_layer_gemm_and_aggregate_device_row_count(dev):
    """M_dev / nS_dev below the capacity: the first rows equal a call of that size, the rest stay untouched."""
    from paper_2101_07706_amd import csgs
    rng = np.random.default_rng(8)
    for M, K, N, m in [(700, 96, 80, 389), (700, 100, 80, 389), (1024, 256, 256, 1000), (1024, 68, 256, 3),
                       (16512, 256, 256, 16001), (16384, 100, 256, 9000)]:
        _gemm_device_row_count(dev, rng, M, K, N, m)
    M, K, N, m = 700, 96, 80, 389
    Z = rng.standard_normal((M, K)).astype(np.float32)
    W = rng.standard_normal((K, N)).astype(np.float32)
    Zd, Wd = torch.from_numpy(Z).to(dev), torch.from_numpy(W).to(dev)
    Zd[m:] = float("nan")          # rows beyond the count may be read; what they hold must reach nothing
    Zd[m + 1::3] = float("inf")
    H = torch.full((M, N), float("nan"), dtype=torch.float32, device=dev)
    cnt = torch.tensor([m], dtype=torch.int32, device=dev)
    csgs.csgs_layer_gemm(Zd, Wd, H, M_dev=cnt)
    torch.cuda.synchronize()
    chain.assert_close(H[:m].cpu().numpy(), oracle.layer_gemm(Z[:m], W), chain.RTOL, chain.ATOL, "H with M_dev")
    assert bool(torch.isnan(H[m:]).all())
    # aggregation: random CSR with M rows over 300 input rows
    deg = rng.integers(0, 70, M)
    rp = np.zeros(M + 1, np.int32)
    np.cumsum(deg, out=rp[1:])
    col = np.concatenate([np.sort(rng.choice(300, d, replace=False)) for d in deg]).astype(np.int32)
    val = rng.standard_normal(len(col)).astype(np.float32)
    X = rng.standard_normal((300, K)).astype(np.float32)
    Zo = torch.full((M, K), float("nan"), dtype=torch.float32, device=dev)
    csgs.csgs_aggregate(torch.from_numpy(rp).to(dev), torch.from_numpy(col).to(dev), torch.from_numpy(val).to(dev),
                        None, torch.from_numpy(X).to(dev), None, None, True, Zo, nS_dev=cnt)
    torch.cuda.synchronize()
    want = oracle.aggregate(rp[:m + 1], col[:rp[m]], val[:rp[m]], X, relu_on_input=True)
    chain.assert_close(Zo[:m].cpu().numpy(), want, chain.RTOL, chain.ATOL, "Z with nS_dev")
    assert bool(torch.isnan(Zo[m:]).all())


def test_recorded_plan_replays_calls(dev):
    """csgs.record(): wrapper calls made while recording are not enqueued; Plan.run() issues them with
    the arguments marshalled once, boxes (batch pointer, iteration number) read at every run."""
    import ctypes as C
    from paper_2101_07706_amd import csgs, pipeline
    g = SmallGraph(1500, 9, seed=21, lo=200, hi=700)
    rng = np.random.default_rng(2)
    B = 96
    batches = [rng.permutation(1500)[:120].astype(np.int32) for _ in range(3)]
    dg = pipeline.DeviceGraph(g, dev)
    ws = pipeline.Workspace(g.n_nodes, 120, B, g.nnz, dev)
    lb = pipeline.LayerBuffers(120, B, g.n_nodes, g.nnz, dg.n_parts, dev)
    Sd = [torch.from_numpy(b).to(dev) for b in batches]
    S_box, it_box = csgs.DevicePtr(120), C.c_uint64(0)
    lb.n_next.fill_(-5)
    with csgs.record() as plan:
        pipeline.sample_step(dg, ws, S_box, 2.0, B, 77, it_box, 1, lb)
    torch.cuda.synchronize()
    assert int(lb.n_next.item()) == -5 and len(plan.calls) == 2, "recording must not enqueue anything"
    for it, b in enumerate(batches):
        S_box.value, it_box.value = Sd[it].data_ptr(), it
        plan.run()
        torch.cuda.synchronize()
        pr = oracle.build_probs(g, b, 2.0)
        sm = oracle.sample_layer(g, b, pr, B, 77, it, 1)
        assert int(lb.status.item()) == 0 and int(lb.n_next.item()) == sm.n_next
        np.testing.assert_array_equal(lb.S_next[:sm.n_next].cpu().numpy(), sm.S_next)
        np.testing.assert_array_equal(lb.adj_rowptr[:121].cpu().numpy(), sm.adj_rowptr)
        np.testing.assert_array_equal(lb.adj_col[:sm.adj_nnz].cpu().numpy(), sm.adj_col)


def test_step_replayed_from_a_hip_graph(dev):
    """A two-layer step captured once into a HIP graph and replayed for several batches and iteration
    numbers (passed through device memory), with eager library work on the same workspace and
    synchronisations between the replays: every replay equals the oracle."""
    from paper_2101_07706_amd import pipeline
    g = SmallGraph(4000, 14, seed=31, lo=1000, hi=2400)
    rng = np.random.default_rng(6)
    F, Fh, B, nS0, seed = 32, 24, 200, 150, 4321
    X = rng.standard_normal((g.n_nodes, F)).astype(np.float32)
    Ws = [synth.glorot_uniform(F, Fh, 1), synth.glorot_uniform(Fh, 8, 2)]
    dg = pipeline.DeviceGraph(g, dev)
    ws = pipeline.Workspace(g.n_nodes, max(nS0, B), B, g.nnz, dev)
    lbs = [pipeline.LayerBuffers(max(nS0, B), B, g.n_nodes, g.nnz, dg.n_parts, dev) for _ in range(2)]
    Xd = torch.from_numpy(X).to(dev)
    Wd = [torch.from_numpy(W).to(dev) for W in Ws]
    S0buf = torch.zeros(nS0, dtype=torch.int32, device=dev)
    iter_dev = torch.zeros(1, dtype=torch.int64, device=dev)
    staged = torch.zeros((B, F), dtype=torch.float32, device=dev)
    Z = [torch.zeros((nS0, Fh), dtype=torch.float32, device=dev), torch.zeros((B, F), dtype=torch.float32, device=dev)]
    H = [torch.zeros((nS0, 8), dtype=torch.float32, device=dev), torch.zeros((B, Fh), dtype=torch.float32, device=dev)]

    def enqueue():
        pipeline.sample_step(dg, ws, S0buf, 3.0, B, seed, 0, 0, lbs[0], iter_dev=iter_dev)
        pipeline.sample_step(dg, ws, lbs[0].S_next, 3.0, B, seed, 0, 1, lbs[1], nS_dev=lbs[0].n_next, iter_dev=iter_dev)
        pipeline.stage_remote_rows(lbs[1], Xd, staged)
        pipeline.compute_step(lbs[1], B, Xd[g.local_lo:g.local_hi], staged, True, False, Wd[0], Z[1], H[1], nS_dev=lbs[0].n_next)
        pipeline.compute_step(lbs[0], nS0, H[1], None, False, True, Wd[1], Z[0], H[0])

    batches = [rng.permutation(np.arange(g.local_lo, g.local_hi))[:nS0].astype(np.int32) for _ in range(4)]
    S0buf.copy_(torch.from_numpy(batches[0]).to(dev))
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):      # one eager pass before capture
        enqueue()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        enqueue()
    torch.cuda.synchronize()
    for rep, (b, it) in enumerate(zip(batches, [5, 5, 9, 2 ** 33 + 1])):
        S0buf.copy_(torch.from_numpy(b).to(dev))
        iter_dev.fill_(it)
        for lb in lbs:
            lb.status.zero_()
        if rep % 2 == 1:   # eager library work on the same workspace between replays
            scratch = pipeline.LayerBuffers(max(nS0, B), B, g.n_nodes, g.nnz, dg.n_parts, dev)
            pipeline.sample_step(dg, ws, S0buf, 1.0, B, 1, 0, 0, scratch)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        osteps = chain.oracle_chain(g, X, Ws, b, 3.0, B, seed, it)
        n1 = osteps[0].sm.n_next
        gsteps = [SimpleNamespaceLike(S=S0buf, lb=lbs[0], n_next=int(lbs[0].n_next.item()), status=int(lbs[0].status.item()),
                                      Z=Z[0], H=H[0]),
                  SimpleNamespaceLike(S=lbs[0].S_next[:n1], lb=lbs[1], n_next=int(lbs[1].n_next.item()),
                                      status=int(lbs[1].status.item()), Z=Z[1][:n1], H=H[1][:n1])]
        worst = chain.compare_chain(osteps, gsteps)
        say(f"[graph] replay {rep}: iter {it}, n' {[o.sm.n_next for o in osteps]}, worst err/tol {max(worst.values()):.3f}")


class SimpleNamespaceLike:
    def __init__(self, **kw):
        self.__dict__.update(kw)


def test_subgraph_sampler_without_host_reads(dev):
    """Subgraph sampler with the number of drawn nodes left on the device: rows of the sampled operator
    = S_next at its capacity B, n_rows_dev = n_next; aggregation and GEMM with the same device count."""
    from paper_2101_07706_amd import csgs, pipeline
    g = SmallGraph(2500, 11, seed=8, lo=300, hi=1300)
    rng = np.random.default_rng(3)
    F, B, seed, skew = 24, 380, 17, 2.0
    X = rng.standard_normal((g.n_nodes, F)).astype(np.float32)
    W = synth.glorot_uniform(F, 12, 5)
    n = g.n_nodes
    rows_all = np.arange(n, dtype=np.int32)
    pr = oracle.build_probs(g, rows_all, skew)
    dr = oracle.draw_nodes(pr, B, seed, 4, 0)
    adj = oracle.sampled_adjacency(g, dr.S_next, dr)
    rc = oracle.remote_count(dr.S_next, g.local_lo, g.local_hi, g.part_bounds)
    Zo = oracle.aggregate(adj.adj_rowptr, adj.adj_col, adj.adj_val, X[g.local_lo:g.local_hi], X[rc.remote_ids], rc.src_row)
    Ho = oracle.layer_gemm(Zo, W)

    dg = pipeline.DeviceGraph(g, dev)
    ws = pipeline.Workspace(n, n, B, g.nnz, dev)
    lb = pipeline.LayerBuffers(n, B, n, int(g.nnz), dg.n_parts, dev)
    Xd, Wd = torch.from_numpy(X).to(dev), torch.from_numpy(W).to(dev)
    staged = torch.zeros((B, F), dtype=torch.float32, device=dev)
    Zd = torch.full((B, F), float("nan"), dtype=torch.float32, device=dev)
    Hd = torch.full((B, 12), float("nan"), dtype=torch.float32, device=dev)
    lb.adj_rowptr.fill_(-3)
    csgs.csgs_build_probs(dg.c, torch.from_numpy(rows_all).to(dev), skew, lb.cand_id, lb.cand_w, lb.cdf, lb.q, lb.stats, ws.desc,
                          lb.status)
    csgs.csgs_draw_nodes(n, lb.cand_id, lb.cdf, lb.stats, B, seed, 4, 0, lb.S_next, lb.mult, lb.p_incl, lb.n_next, ws.desc, lb.status)
    csgs.csgs_sampled_adjacency(dg.c, lb.S_next, lb.adj_rowptr[:B + 1], lb.adj_col, lb.adj_val, lb.adj_nnz, ws.desc, lb.status,
                                n_rows_dev=lb.n_next)
    csgs.csgs_remote_count(lb.S_next, lb.n_next, g.local_lo, g.local_hi, dg.part_bounds, lb.remote_total, lb.per_part,
                           lb.src_row, lb.remote_ids)
    pipeline.stage_remote_rows(lb, Xd, staged)
    pipeline.compute_step(lb, B, Xd[g.local_lo:g.local_hi], staged, True, False, Wd, Zd, Hd, nS_dev=lb.n_next)
    torch.cuda.synchronize()
    m = int(lb.n_next.item())
    assert int(lb.status.item()) == 0 and m == dr.n_next and m < B
    np.testing.assert_array_equal(lb.adj_rowptr[:m + 1].cpu().numpy(), adj.adj_rowptr)
    assert bool((lb.adj_rowptr[m + 1:B + 1] == -3).all())
    np.testing.assert_array_equal(lb.adj_col[:adj.adj_nnz].cpu().numpy(), adj.adj_col)
    chain.assert_close(lb.adj_val[:adj.adj_nnz].cpu().numpy(), adj.adj_val, chain.P_RTOL, 0.0, "adj_val")
    chain.assert_close(Zd[:m].cpu().numpy(), Zo, chain.RTOL, chain.ATOL, "Z")
    chain.assert_close(Hd[:m].cpu().numpy(), Ho, chain.RTOL, chain.ATOL, "H")
    assert bool(torch.isnan(Zd[m:]).all()) and bool(torch.isnan(Hd[m:]).all())


def test_four_call_sequences_side_by_side(dev):
    """Four sampling call sequences on four workspaces and four streams at once (the documented limit
    of concurrent sequences): each gives the result of running alone."""
    from paper_2101_07706_amd import pipeline
    cfg, g, X, Ws, _ = chain.config_inputs("medium")
    dg = pipeline.DeviceGraph(g, dev)
    B = cfg.samples
    batches = [synth.make_batch(g, cfg.batch, cfg.seed, it) for it in range(4)]
    Sd = [torch.from_numpy(b).to(dev) for b in batches]
    wss = [pipeline.Workspace(g.n_nodes, max(cfg.batch, B), B, g.nnz, dev) for _ in range(4)]
    lbs = [[pipeline.LayerBuffers(max(cfg.batch, B), B, g.n_nodes, 4_000_000, dg.n_parts, dev) for _ in range(2)] for _ in range(4)]
    streams = [torch.cuda.Stream() for _ in range(4)]
    torch.cuda.synchronize()
    for rep in range(3):
        for j in range(4):
            pipeline.sample_step(dg, wss[j], Sd[j], cfg.skew, B, 99, rep, 0, lbs[j][0], stream=streams[j])
            pipeline.sample_step(dg, wss[j], lbs[j][0].S_next, cfg.skew, B, 99, rep, 1, lbs[j][1], stream=streams[j],
                                 nS_dev=lbs[j][0].n_next)
    torch.cuda.synchronize()
    for j in range(4):
        S = batches[j]
        for l in range(2):
            pr = oracle.build_probs(g, S, cfg.skew)
            sm = oracle.sample_layer(g, S, pr, B, 99, 2, l)
            lb = lbs[j][l]
            assert int(lb.status.item()) == 0 and int(lb.n_next.item()) == sm.n_next
            np.testing.assert_array_equal(lb.S_next[:sm.n_next].cpu().numpy(), sm.S_next)
            np.testing.assert_array_equal(lb.adj_rowptr[:len(S) + 1].cpu().numpy(), sm.adj_rowptr)
            np.testing.assert_array_equal(lb.adj_col[:sm.adj_nnz].cpu().numpy(), sm.adj_col)
            S = sm.S_next


# ---------------------------------------------------------------- gradients of a layer
def _scratch(nbytes, dev):
    return torch.empty(max(nbytes, 256) // 8 + 32, dtype=torch.int64, device=dev)


@pytest.mark.parametrize("M,K,N", [(1, 1, 1), (33, 17, 5), (700, 96, 80), (4096, 300, 512), (8192, 256, 256), (7001, 100, 256),
                                   (5000, 256, 47)])
def test_layer_gemm_gradients(dev, M, K, N):
    from paper_2101_07706_amd import csgs
    rng = np.random.default_rng(M + K + N)
    Z = rng.standard_normal((M, K)).astype(np.float32)
    G = rng.standard_normal((M, N)).astype(np.float32)
    W = rng.standard_normal((K, N)).astype(np.float32)
    Zd, Gd, Wd = (torch.from_numpy(a).to(dev) for a in (Z, G, W))
    dW = torch.full((K, N), float("nan"), dtype=torch.float32, device=dev)
    dZ = torch.full((M, K), float("nan"), dtype=torch.float32, device=dev)
    scratch = _scratch(csgs.csgs_layer_gemm_grad_w_scratch_bytes(M, K, N), dev)
    csgs.csgs_layer_gemm_grad_w(Zd, Gd, dW, scratch)
    csgs.csgs_layer_gemm_grad_z(Gd, Wd, dZ)
    torch.cuda.synchronize()
    # identical inputs and double accumulation on both sides: the stated tolerance as it stands
    chain.assert_close(dW.cpu().numpy(), oracle.layer_gemm_grad_w(Z, G), chain.RTOL, chain.ATOL, "dW")
    chain.assert_close(dZ.cpu().numpy(), oracle.layer_gemm_grad_z(G, W), chain.RTOL, chain.ATOL, "dZ")
    if M > 40:   # device row count below the capacity
        m = M - 37
        cnt = torch.tensor([m], dtype=torch.int32, device=dev)
        dW.fill_(float("nan"))
        dZ.fill_(float("nan"))
        Zd[m:] = float("nan")      # rows beyond the count: never summed into dW, never reach a written row of dZ
        Gd[m:] = float("inf")
        csgs.csgs_layer_gemm_grad_w(Zd, Gd, dW, scratch, M_dev=cnt)
        csgs.csgs_layer_gemm_grad_z(Gd, Wd, dZ, M_dev=cnt)
        torch.cuda.synchronize()
        chain.assert_close(dW.cpu().numpy(), oracle.layer_gemm_grad_w(Z[:m], G[:m]), chain.RTOL, chain.ATOL, "dW with M_dev")
        chain.assert_close(dZ[:m].cpu().numpy(), oracle.layer_gemm_grad_z(G[:m], W), chain.RTOL, chain.ATOL, "dZ with M_dev")
        assert bool(torch.isnan(dZ[m:]).all())


@pytest.mark.parametrize("nS,nc,F,maxdeg,relu", [(1, 1, 4, 1, False), (300, 257, 64, 9, True), (2048, 1500, 256, 40, True),
                                                 (500, 64, 100, 64, False), (3000, 3000, 33, 6, True)])
def test_aggregate_gradient(dev, nS, nc, F, maxdeg, relu):
    from paper_2101_07706_amd import csgs
    rng = np.random.default_rng(nS + nc + F)
    deg = rng.integers(0, min(maxdeg, nc) + 1, nS)
    if nS > 100:
        deg[7] = min(nc, 700)                # a hub row
    rp = np.zeros(nS + 1, np.int32)
    np.cumsum(deg, out=rp[1:])
    col = np.concatenate([np.sort(rng.choice(nc, d, replace=False)) for d in deg] + [np.zeros(0, np.int64)]).astype(np.int32)
    val = rng.standard_normal(len(col)).astype(np.float32)
    dZ = rng.standard_normal((nS, F)).astype(np.float32)
    Hp = rng.standard_normal((nc, F)).astype(np.float32)
    cap = max(len(col), 1) + 5
    rpd, cold, vald = torch.from_numpy(rp).to(dev), torch.zeros(cap, dtype=torch.int32, device=dev), torch.zeros(cap, device=dev)
    cold[:len(col)] = torch.from_numpy(col).to(dev)
    vald[:len(col)] = torch.from_numpy(val).to(dev)
    dH = torch.full((nc, F), float("nan"), dtype=torch.float32, device=dev)
    scratch = _scratch(csgs.csgs_aggregate_grad_scratch_bytes(nc, cap), dev)
    n_next = torch.tensor([nc], dtype=torch.int32, device=dev)
    csgs.csgs_aggregate_grad(rpd, cold, vald, n_next, torch.from_numpy(dZ).to(dev), torch.from_numpy(Hp).to(dev) if relu else None,
                             dH, scratch)
    torch.cuda.synchronize()
    want = oracle.aggregate_grad(rp, col, val, nc, dZ, Hp if relu else None)
    chain.assert_close(dH.cpu().numpy(), want, chain.RTOL, chain.ATOL, "dH_prev")
    # twice in a row on the same scratch (the counters are re-zeroed by the call itself): the same bits, every
    # column being summed in ascending row order whatever order its entries arrived in
    first = dH.clone()
    dH.fill_(float("nan"))
    csgs.csgs_aggregate_grad(rpd, cold, vald, n_next, torch.from_numpy(dZ).to(dev), torch.from_numpy(Hp).to(dev) if relu else None,
                             dH, scratch)
    torch.cuda.synchronize()
    chain.assert_close(dH.cpu().numpy(), want, chain.RTOL, chain.ATOL, "dH_prev, second call")
    assert torch.equal(first, dH), "two calls of the aggregation gradient differ in some bit"


def _rel_frobenius(got, want):
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    return float(np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-300))


@pytest.mark.parametrize("name", ["tiny", "medium", "mid", "large"])
def test_backward_chain(dev, name):
    """Forward with device-side row counts, then the gradients of every layer bottom-up from a random
    dL/dH of the top layer, all row counts left on the device.  Every gradient call is checked against
    the oracle function applied to the very arrays the call read (downloaded), at the stated tolerance.
    The oracle's own chain starts from forward results that differ from the device's in the last bit of a
    few entries, which a near-cancelling gradient entry can amplify beyond 1e-5 absolute, so chain
    against chain is compared in the Frobenius norm."""
    from paper_2101_07706_amd import csgs
    if name == "large":
        cfg, g, X, Ws, _ = cached_inputs(name)
        S0 = synth.make_batch(g, cfg.batch, cfg.seed, 0)
    else:
        cfg, g, X, Ws, S0 = chain.config_inputs(name)
    bf16 = cfg.feat_dtype == "bf16"
    B, M = cfg.samples, len(Ws)
    say(f"[{name}] backward chain: forward")
    osteps = chain.oracle_chain(g, X, Ws, S0, cfg.skew, B, 1234 + cfg.seed, 0, bf16)
    gsteps, _ = chain.gpu_chain(g, X, Ws, S0, cfg.skew, B, 1234 + cfg.seed, 0, bf16, device_counts=True,
                                adj_cap=min(g.nnz, 1 << 24))
    chain.compare_chain(osteps, gsteps)
    rng = np.random.default_rng(9)
    G0 = rng.standard_normal(osteps[0].H.shape).astype(np.float32)
    # oracle: layer 0 is the top (its rows are the batch); dL/dH of layer l+1 comes from layer l's input gradient
    Go, want = G0, []
    for l in range(M):
        o = osteps[l]
        W = Ws[M - 1 - l]
        dW = oracle.layer_gemm_grad_w(o.Z, Go)
        dZ = oracle.layer_gemm_grad_z(Go, W)
        dH = None
        if l < M - 1:
            dH = oracle.aggregate_grad(o.sm.adj_rowptr, o.sm.adj_col, o.sm.adj_val, o.sm.n_next, dZ, osteps[l + 1].H)
        want.append((dW, dZ, dH))
        Go = dH
    # GPU: capacity-sized arrays, device counts
    Gd = torch.from_numpy(G0).to(dev)
    worst, chain_err = 0.0, 0.0
    for l in range(M):
        say(f"[{name}] backward chain: layer {l}")
        gs, lb = gsteps[l], gsteps[l].lb
        nS_cap = len(S0) if l == 0 else B
        nS_dev = None if l == 0 else gsteps[l - 1].lb.n_next
        W = Ws[M - 1 - l]
        Wd = torch.from_numpy(W).to(dev)
        K, N = Wd.shape
        Zfull = gs.Z._base if gs.Z._base is not None else gs.Z          # the capacity-sized buffer behind the view
        Zfull = Zfull[:nS_cap]
        Gfull = torch.zeros((nS_cap, N), dtype=torch.float32, device=dev)
        Gfull[:Gd.shape[0]] = Gd
        dW = torch.full((K, N), float("nan"), dtype=torch.float32, device=dev)
        dZ = torch.full((nS_cap, K), float("nan"), dtype=torch.float32, device=dev)
        sw = _scratch(csgs.csgs_layer_gemm_grad_w_scratch_bytes(nS_cap, K, N), dev)
        csgs.csgs_layer_gemm_grad_w(Zfull, Gfull, dW, sw, M_dev=nS_dev)
        csgs.csgs_layer_gemm_grad_z(Gfull, Wd, dZ, M_dev=nS_dev)
        torch.cuda.synchronize()
        n_rows = len(osteps[l].S)
        Z_in, G_in = Zfull[:n_rows].cpu().numpy(), Gfull[:n_rows].cpu().numpy()
        worst = max(worst, chain.assert_close(dW.cpu().numpy(), oracle.layer_gemm_grad_w(Z_in, G_in), chain.RTOL, chain.ATOL,
                                              f"layer {l} dW"))
        worst = max(worst, chain.assert_close(dZ[:n_rows].cpu().numpy(), oracle.layer_gemm_grad_z(G_in, W), chain.RTOL, chain.ATOL,
                                              f"layer {l} dZ"))
        assert bool(torch.isnan(dZ[n_rows:]).all())
        chain_err = max(chain_err, _rel_frobenius(dW.cpu().numpy(), want[l][0]), _rel_frobenius(dZ[:n_rows].cpu().numpy(), want[l][1]))
        if l < M - 1:
            Hp = gsteps[l + 1].H
            Hp = (Hp._base if Hp._base is not None else Hp)[:B]
            dH = torch.full((B, K), float("nan"), dtype=torch.float32, device=dev)
            sa = _scratch(csgs.csgs_aggregate_grad_scratch_bytes(B, lb.adj_col.numel()), dev)
            csgs.csgs_aggregate_grad(lb.adj_rowptr[:nS_cap + 1], lb.adj_col, lb.adj_val, lb.n_next, dZ, Hp, dH, sa, nS_dev=nS_dev)
            torch.cuda.synchronize()
            m = osteps[l].sm.n_next
            nnz = osteps[l].sm.adj_nnz
            ref = oracle.aggregate_grad(lb.adj_rowptr[:n_rows + 1].cpu().numpy(), lb.adj_col[:nnz].cpu().numpy(),
                                        lb.adj_val[:nnz].cpu().numpy(), m, dZ[:n_rows].cpu().numpy(), Hp[:m].cpu().numpy())
            worst = max(worst, chain.assert_close(dH[:m].cpu().numpy(), ref, chain.RTOL, chain.ATOL, f"layer {l} dH_prev"))
            assert bool(torch.isnan(dH[m:]).all())
            chain_err = max(chain_err, _rel_frobenius(dH[:m].cpu().numpy(), want[l][2]))
            # bit-reproducible: a second call on the same scratch gives the same bits
            dH2 = torch.full((B, K), float("nan"), dtype=torch.float32, device=dev)
            csgs.csgs_aggregate_grad(lb.adj_rowptr[:nS_cap + 1], lb.adj_col, lb.adj_val, lb.n_next, dZ, Hp, dH2, sa, nS_dev=nS_dev)
            torch.cuda.synchronize()
            assert torch.equal(dH[:m], dH2[:m]), f"layer {l}: two calls of the aggregation gradient differ"
            Gd = dH[:m]
    assert chain_err < 1e-6, f"gradient chain against the oracle's chain: relative Frobenius error {chain_err:.3e}"
    say(f"[{name}] backward chain: {M} layers, worst err/tol per call {worst:.3f}, chain against chain {chain_err:.2e} (Frobenius), "
        f"|dW| max {[float(np.abs(w[0]).max()) for w in want]}")


def test_calibration_kernels(dev):
    """The two yardstick kernels do what their byte / update counts assume."""
    from paper_2101_07706_amd import csgs
    src = torch.arange(1 << 16, dtype=torch.int64, device=dev)
    dst = torch.zeros_like(src)
    csgs.csgs_calib_copy(dst, src)
    table = torch.zeros(1000, dtype=torch.int64, device=dev)
    csgs.csgs_calib_atomics(table, 123457)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)
    assert int(table.sum().item()) == 123457 and int(table.min().item()) > 0
    # matrix-core yardstick: the sums say how many instructions ran.  Lane l feeds A[l % 16][l // 16] and
    # B[l // 16][l % 16] of a 16 x 16 x 4 product; the kernel adds up every accumulator element
    iters = 3
    sink = torch.zeros(csgs.CALIB_MFMA_BLOCKS * 256, dtype=torch.float64, device=dev)
    flops = csgs.csgs_calib_mfma_f64(sink, iters)
    torch.cuda.synchronize()
    assert flops == csgs.CALIB_MFMA_BLOCKS * 4 * 64 * 2048 * iters
    lane = np.arange(64)
    m, k = lane % 16, lane // 16
    A0 = np.zeros((16, 4)); A1 = np.zeros((16, 4)); Bm = np.zeros((4, 16))
    A0[m, k] = 1.0 / (lane + 1); A1[m, k] = 1.0 / (lane + 65); Bm[k, m] = 1.0 / (lane + 129)
    per_wave = 4 * 8 * iters * float((A0 @ Bm).sum() + (A1 @ Bm).sum())
    got = sink.cpu().numpy().reshape(-1, 64).sum(axis=1)
    np.testing.assert_allclose(got, per_wave, rtol=1e-12)
    csgs.csgs_calib_mfma_f64(sink, iters, from_lds=True)
    torch.cuda.synchronize()
    got = sink.cpu().numpy().reshape(-1, 256)
    assert np.isfinite(got).all() and (got > 0).all() and (got == got[0]).all()
    with pytest.raises(RuntimeError):
        csgs.csgs_calib_mfma_f64(sink[:1000], iters)
    # random-lookup yardstick: reads the entries the atomic-add yardstick updates, so with table[i] = 1 before ...
    table = torch.zeros(1000, dtype=torch.int64, device=dev)
    csgs.csgs_calib_atomics(table, 54321)
    lsink = torch.zeros(1 << 22, dtype=torch.int64, device=dev)
    ones = torch.ones(1000, dtype=torch.int64, device=dev)
    csgs.csgs_calib_lookups(ones, 54321, lsink)
    torch.cuda.synchronize()
    assert int(lsink.sum().item()) == 54321                      # ... every read is counted once
    csgs.csgs_calib_lookups(torch.arange(1000, dtype=torch.int64, device=dev), 54321, lsink)
    torch.cuda.synchronize()
    # and the entries read are those the updates went to: sum of index * (updates of that entry)
    assert int(lsink.sum().item()) == int((table * torch.arange(1000, dtype=torch.int64, device=dev)).sum().item())


@pytest.mark.parametrize("scan_mode", [1, 2])
def test_failed_waits_end_normally_and_are_reported(dev, scan_mode):
    """Timeout path of the waits between blocks, forced from the host: with a poll limit of zero a
    wait that is not satisfied at once gives up.  Every kernel must still end (no hang, all accesses
    in bounds), the status word must say so, and after csgs_workspace_init the same workspace must
    give exact results again.  Both forms of the weight scan (the owner blocks of the second wait for
    the chunk blocks)."""
    from paper_2101_07706_amd import csgs, pipeline
    cfg, g, X, Ws, S0 = chain.config_inputs("medium")
    dg = pipeline.DeviceGraph(g, dev)
    B = cfg.samples
    ws = pipeline.Workspace(g.n_nodes, max(len(S0), B), B, g.nnz, dev, scan_mode=scan_mode)
    lbs = [pipeline.LayerBuffers(max(len(S0), B), B, g.n_nodes, 4_000_000, dg.n_parts, dev) for _ in range(2)]
    Sd = torch.from_numpy(S0).to(dev)
    Xd = torch.from_numpy(X).to(dev)
    Z = torch.zeros((B, X.shape[1]), dtype=torch.float32, device=dev)
    staged = torch.zeros((B, X.shape[1]), dtype=torch.float32, device=dev)

    def run(it):
        for lb in lbs:
            lb.status.zero_()
        pipeline.sample_step(dg, ws, Sd, cfg.skew, B, 7, it, 0, lbs[0])
        pipeline.sample_step(dg, ws, lbs[0].S_next, cfg.skew, B, 7, it, 1, lbs[1], nS_dev=lbs[0].n_next)
        pipeline.stage_remote_rows(lbs[1], Xd, staged)
        csgs.csgs_aggregate(lbs[1].adj_rowptr[:B + 1], lbs[1].adj_col, lbs[1].adj_val, lbs[1].n_next,
                            Xd[g.local_lo:g.local_hi], staged, lbs[1].src_row, False, Z, nS_dev=lbs[0].n_next)
        torch.cuda.synchronize()
        return [int(lb.status.item()) for lb in lbs]

    def check_exact(it):
        S = S0
        for l in range(2):
            pr = oracle.build_probs(g, S, cfg.skew)
            sm = oracle.sample_layer(g, S, pr, B, 7, it, l)
            assert int(lbs[l].n_next.item()) == sm.n_next
            np.testing.assert_array_equal(lbs[l].S_next[:sm.n_next].cpu().numpy(), sm.S_next)
            np.testing.assert_array_equal(lbs[l].adj_rowptr[:len(S) + 1].cpu().numpy(), sm.adj_rowptr)
            S = sm.S_next

    assert run(0) == [0, 0]
    check_exact(0)
    csgs.csgs_workspace_wait_limit(ws.desc, 0)
    seen = 0
    for it in range(1, 4):
        st = run(it)            # must return: that is the test
        seen |= st[0] | st[1]
        csgs.csgs_workspace_init(ws.desc)
        csgs.csgs_workspace_wait_limit(ws.desc, 0)
    say(f"[waits] status bits seen with a poll limit of zero: {seen:#x}")
    assert seen & csgs.ST_INTERNAL, "no wait gave up although none may poll"
    csgs.csgs_workspace_init(ws.desc)            # also puts the built-in limit back
    assert run(9) == [0, 0]
    check_exact(9)
