"""Buffer management and call order for a sampled mini-batch on one GPU.

Nothing here computes: it allocates torch tensors as device memory, uploads
the synthetic inputs, and issues the library calls in the order the method
prescribes (top-down sampling, Sections 4.1-4.2; bottom-up layer compute,
Eq. 1).  Staging the feature rows of sampled remote nodes stands in for the
exchange between GPUs (Section 3, "Communication of Feature Vectors").
"""
from __future__ import annotations

import ctypes as C
from types import SimpleNamespace

import numpy as np
import torch

from . import csgs


class DeviceGraph:
    def __init__(self, g, device="cuda:0"):
        self.device = torch.device(device)
        self.n_nodes = g.n_nodes
        self.rowptr = torch.from_numpy(g.rowptr).to(self.device)
        self.colidx = torch.from_numpy(g.colidx).to(self.device)
        self.val = torch.from_numpy(g.val).to(self.device)
        self.local_lo, self.local_hi = g.local_lo, g.local_hi
        self.part_bounds = torch.from_numpy(np.ascontiguousarray(g.part_bounds, np.int32)).to(self.device)
        self.n_parts = len(g.part_bounds) - 1
        self.c = csgs.make_graph(self.rowptr, self.colidx, self.val, g.local_lo, g.local_hi, g.rownorm2_max)


class Workspace:
    def __init__(self, n_nodes, nS_max, B_max, edges_max, device):
        nbytes = csgs.csgs_workspace_bytes(n_nodes, nS_max, B_max, edges_max)
        assert nbytes > 0
        self.buf = torch.empty(nbytes // 8, dtype=torch.int64, device=device)
        assert self.buf.data_ptr() % 256 == 0
        self.desc = csgs.make_workspace(self.buf, n_nodes, nS_max, B_max, edges_max)
        csgs.csgs_workspace_init(self.desc)


class LayerBuffers:
    """Outputs of one sampling step (one GCN layer)."""

    def __init__(self, nS_max, B, cand_cap, adj_cap, n_parts, device):
        i32, i64, f32 = torch.int32, torch.int64, torch.float32
        e = lambda n, dt: torch.empty(max(int(n), 1), dtype=dt, device=device)
        self.cand_id, self.cand_w, self.cdf, self.q = e(cand_cap, i32), e(cand_cap, i64), e(cand_cap, i64), e(cand_cap, f32)
        self.stats = torch.zeros(8, dtype=i64, device=device)
        self.S_next, self.mult, self.p_incl = e(B, i32), e(B, i32), e(B, f32)
        self.n_next = torch.zeros(1, dtype=i32, device=device)
        self.adj_rowptr, self.adj_col, self.adj_val = e(nS_max + 1, i32), e(adj_cap, i32), e(adj_cap, f32)
        self.adj_nnz = torch.zeros(1, dtype=i64, device=device)
        self.remote_total = torch.zeros(1, dtype=i64, device=device)
        self.per_part = torch.zeros(n_parts, dtype=i64, device=device)
        self.src_row, self.remote_ids = e(B, i32), e(B, i32)
        self.status = torch.zeros(1, dtype=i32, device=device)
        self.B = B
        self.remote = None     # csgs_remote_out over these buffers, made on first use (needs the partition bounds)

    def stats_host(self):
        raw = self.stats.cpu().numpy().tobytes()
        s = csgs.ProbStats.from_buffer_copy(raw)
        return SimpleNamespace(n_cand=s.n_cand, n_local=s.n_local, n_remote=s.n_remote,
                               edges_scanned=s.edges_scanned, w_local=s.w_local, w_remote=s.w_remote,
                               total=s.total, shift=s.shift, skew_fx=s.skew_fx)


def sample_step(dg, ws, S, skew, B, seed, it, layer, lb, stream=None, want_q=True, auto_D=None, nS_dev=None,
                iter_dev=None, fuse_remote=True):
    """csgs_build_probs -> csgs_sample_layer (-> csgs_remote_count) for the rows S (device int32).
    auto_D: take the skew from Theorem 1 with this constant; `skew` is then its upper bound.
    nS_dev: device int32 with the number of rows of S to use (the previous layer's n_next), so that
    the host need not wait for it; S is then the whole capacity-sized array.
    S None: the rows are the node set the previous csgs_sample_layer on `ws` sampled (it has prepared
    their offsets); B must be the same as in that call.
    iter_dev: device uint64 with the iteration number (for replayed call sequences).
    fuse_remote: let csgs_sample_layer write the remote split (one launch less); False: call
    csgs_remote_count separately."""
    nS = S.numel() if S is not None else B       # S None: rows = the previous layer's sampled set, capacity B
    q = lb.q if want_q else None
    if auto_D is None:
        csgs.csgs_build_probs(dg.c, S, skew, lb.cand_id, lb.cand_w, lb.cdf, q, lb.stats, ws.desc, lb.status, stream,
                              nS_dev=nS_dev, nS=nS)
    else:
        csgs.csgs_build_probs_auto(dg.c, S, auto_D, B, skew, lb.cand_id, lb.cand_w, lb.cdf, q, lb.stats, ws.desc,
                                   lb.status, stream, nS_dev=nS_dev, nS=nS)
    if fuse_remote and lb.remote is None:
        lb.remote = csgs.make_remote_out(dg.local_lo, dg.local_hi, dg.part_bounds, lb.remote_total, lb.per_part, lb.src_row,
                                         lb.remote_ids)
    csgs.csgs_sample_layer(dg.c, S, lb.cand_id, lb.cdf, lb.stats, B, seed, it, layer, lb.S_next, lb.mult,
                           lb.p_incl, lb.n_next, lb.adj_rowptr[:nS + 1], lb.adj_col, lb.adj_val, lb.adj_nnz,
                           ws.desc, lb.status, stream, iter_dev=iter_dev, remote=lb.remote if fuse_remote else None, nS=nS)
    if not fuse_remote:
        csgs.csgs_remote_count(lb.S_next, lb.n_next, dg.local_lo, dg.local_hi, dg.part_bounds, lb.remote_total,
                               lb.per_part, lb.src_row, lb.remote_ids, stream)


def compute_step(lb, nS, X_local, X_remote, use_src_row, relu, W, Z, H, stream=None, nS_dev=None):
    """csgs_aggregate -> csgs_layer_gemm for one layer; Z and H are preallocated [nS, F] / [nS, F_out].
    nS_dev: as in sample_step (nS is then the capacity)."""
    csgs.csgs_aggregate(lb.adj_rowptr[:nS + 1], lb.adj_col, lb.adj_val, lb.n_next, X_local, X_remote,
                        lb.src_row if use_src_row else None, relu, Z, stream, nS_dev=nS_dev)
    csgs.csgs_layer_gemm(Z, W, H, stream, M_dev=nS_dev)


def stage_remote_rows(lb, X, staged, stream=None):
    """Fills `staged` [B, F] with the feature rows of the sampled remote nodes (csgs_gather_rows over the
    request list): the one-GPU stand-in for the exchange between partitions."""
    csgs.csgs_gather_rows(X, lb.remote_ids, lb.remote_total, staged, stream)
