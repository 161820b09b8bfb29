"""Buffer management and call order for a sampled mini-batch on one GPU.

Nothing here computes: it allocates torch tensors as device memory, uploads
the synthetic inputs, and issues the library calls in the order the method
prescribes (top-down sampling, Sections 4.1-4.2; bottom-up layer compute,
Eq. 1).  Staging the feature rows of sampled remote nodes stands in for the
exchange between GPUs (Section 3, the paragraph on the transfer of feature vectors).
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


DEFAULT_SCAN_MODE = 0    # csgs_workspace.scan_mode of new workspaces (tests force either way of the weight scan through it)


class Workspace:
    """Scratch memory of the sampling calls.  n_inst > 1: one workspace per instance back to back;
    calls through it process n_inst instances whose arrays lie inst_stride bytes apart (the layout
    LayerBuffers(n_inst=...) gives them)."""

    def __init__(self, n_nodes, nS_max, B_max, edges_max, device, n_inst=1, inst_stride=0, scan_mode=None):
        nbytes = csgs.csgs_workspace_bytes(n_nodes, nS_max, B_max, edges_max)
        assert nbytes > 0 and nbytes % 256 == 0
        self.bytes_per_inst = nbytes
        self.buf = torch.empty(n_inst * nbytes // 8, dtype=torch.int64, device=device)
        assert self.buf.data_ptr() % 256 == 0
        self.desc = csgs.make_workspace(self.buf, n_nodes, nS_max, B_max, edges_max, n_inst, inst_stride,
                                        DEFAULT_SCAN_MODE if scan_mode is None else scan_mode)
        csgs.csgs_workspace_init(self.desc)


class LayerBuffers:
    """Outputs of one sampling step (one GCN layer), and S0, a place for the rows of the first layer.

    n_inst > 1: the arrays of n_inst instances, every instance's in one contiguous block of
    `stride` bytes with the same layout, so that one library call can fill all of them; the
    attributes are instance 0's arrays (what the calls take), inst(k) gives instance k's."""

    def __init__(self, nS_max, B, cand_cap, adj_cap, n_parts, device, n_inst=1, _share=None, _k=0):
        i32, i64, f32 = torch.int32, torch.int64, torch.float32
        cand_cap, adj_cap = max(int(cand_cap), 1), max(int(adj_cap), 1)
        fields = [("cand_id", cand_cap, i32), ("cand_w", cand_cap, i64), ("cdf", cand_cap, i64), ("q", cand_cap, f32),
                  ("stats", 8, i64), ("S_next", B, i32), ("mult", B, i32), ("p_incl", B, f32), ("n_next", 1, i32),
                  ("adj_rowptr", nS_max + 1, i32), ("adj_col", adj_cap, i32), ("adj_val", adj_cap, f32), ("adj_nnz", 1, i64),
                  ("remote_total", 1, i64), ("per_part", max(n_parts, 1), i64), ("src_row", B, i32), ("remote_ids", B, i32),
                  ("status", 1, i32), ("S0", nS_max, i32)]
        off = 0
        layout = []
        for name, n, dt in fields:
            nbytes = n * torch.empty(0, dtype=dt).element_size()
            layout.append((name, off, nbytes, dt))
            off = (off + nbytes + 255) // 256 * 256
        self.stride = off
        self.n_inst = n_inst
        self._args = (nS_max, B, cand_cap, adj_cap, n_parts, device)
        self.raw = _share if _share is not None else torch.zeros((n_inst, off), dtype=torch.uint8, device=device)
        assert self.raw.data_ptr() % 256 == 0
        row = self.raw[_k]
        for name, o, nbytes, dt in layout:
            setattr(self, name, row[o:o + nbytes].view(dt))
        self.B = B
        self.remote = None     # csgs_remote_out over these buffers, made on first use (needs the partition bounds)

    def inst(self, k):
        """The arrays of instance k (views of the same memory)."""
        assert 0 <= k < self.n_inst
        return LayerBuffers(*self._args, n_inst=self.n_inst, _share=self.raw, _k=k)

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


def instance_strides(lb, x, x_remote, out, n_inst=None):
    """csgs_inst_strides for a compute call on all instances of `lb` at once (or on its first n_inst):
    x / x_remote / out are the byte strides between the instances' input, staged and output matrices
    (0 = shared)."""
    return csgs.InstStrides(lb.n_inst if n_inst is None else n_inst, 0, lb.stride, x, x_remote, out)


def compute_step(lb, nS, X_local, X_remote, use_src_row, relu, W, Z, H, stream=None, nS_dev=None, strides=None, n_inst=None,
                 fused=None):
    """csgs_aggregate -> csgs_layer_gemm for one layer; Z and H are preallocated [nS, F] / [nS, F_out].
    nS_dev: as in sample_step (nS is then the capacity).
    strides = (x, x_remote, z, h) in bytes: all instances of `lb` (or its first n_inst) in the same two
    launches; the tensors passed are instance 0's.
    fused: "h" = one csgs_layer_forward call that leaves Z untouched, "hz" = the same and Z written as well, where
    the input width is one that call takes; the two calls otherwise.  Returns True when the fused call ran."""
    agg = gemm = None
    if fused and csgs.csgs_layer_forward_supported(X_local, X_remote):
        assert fused in ("h", "hz")
        inst, z = None, 0
        if strides is not None:
            x, xr, z, h = strides
            inst = instance_strides(lb, x, xr, h, n_inst)
        csgs.csgs_layer_forward(lb.adj_rowptr[:nS + 1], lb.adj_col, lb.adj_val, lb.n_next, X_local, X_remote,
                                lb.src_row if use_src_row else None, relu, W, H, Z if fused == "hz" else None, stream,
                                nS_dev=nS_dev, inst=inst, z_stride=z)
        return True
    if strides is not None:
        x, xr, z, h = strides
        agg, gemm = instance_strides(lb, x, xr, z, n_inst), instance_strides(lb, z, 0, h, n_inst)
    csgs.csgs_aggregate(lb.adj_rowptr[:nS + 1], lb.adj_col, lb.adj_val, lb.n_next, X_local, X_remote,
                        lb.src_row if use_src_row else None, relu, Z, stream, nS_dev=nS_dev, inst=agg)
    csgs.csgs_layer_gemm(Z, W, H, stream, M_dev=nS_dev, inst=gemm)
    return False


def stage_remote_rows(lb, X, staged, stream=None, out_stride=None, n_inst=None):
    """Fills `staged` [B, F] with the feature rows of the sampled remote nodes (csgs_gather_rows over the
    request list): the one-GPU stand-in for the exchange between partitions.
    out_stride (bytes): all instances of `lb` (or its first n_inst) in one launch, instance k's rows at
    staged + k * out_stride."""
    inst = instance_strides(lb, 0, 0, out_stride, n_inst) if out_stride is not None else None
    csgs.csgs_gather_rows(X, lb.remote_ids, lb.remote_total, staged, stream, inst=inst)
