"""Thin Python binding of libcsgs.so: argument marshalling only.

Same names as the C entry points in include/csgs.h.  Tensors are torch CUDA
(ROCm) tensors used purely as device memory; every step of the method runs in
the library's HIP kernels.  There is no fallback: if the shared library is
missing the import of any entry point raises.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcsgs.so")

OK, EINVAL, EWORKSPACE, EUNSUPPORTED, ERANGE, ELAUNCH = 0, -1, -2, -3, -4, -5
ST_CAND_OVERFLOW, ST_BAD_EDGE_VALUE, ST_EMPTY_CANDIDATES, ST_ADJ_OVERFLOW, ST_BAD_NODE_ID = 1, 2, 4, 8, 16
ST_EDGE_OVERFLOW, ST_INTERNAL = 32, 64
F32, BF16 = 0, 1

EXPORTS = ["csgs_workspace_bytes", "csgs_workspace_clean_bytes", "csgs_workspace_init", "csgs_workspace_wait_limit", "csgs_fixed_point", "csgs_build_probs", "csgs_build_probs_auto",
           "csgs_sample_layer", "csgs_draw_nodes", "csgs_sampled_adjacency", "csgs_remote_count", "csgs_aggregate", "csgs_gather_rows",
           "csgs_layer_gemm", "csgs_aggregate_n", "csgs_gather_rows_n", "csgs_layer_gemm_n", "csgs_layer_forward", "csgs_layer_forward_n", "csgs_layer_forward_supported", "csgs_layer_gemm_grad_w_scratch_bytes", "csgs_layer_gemm_grad_w", "csgs_layer_gemm_grad_w_static", "csgs_layer_gemm_grad_z",
           "csgs_aggregate_grad_scratch_bytes", "csgs_aggregate_grad", "csgs_strerror",
           "csgs_profile_enable", "csgs_profile_kernel_count", "csgs_profile_kernel_name", "csgs_profile_collect", "csgs_profile_samples",
           "csgs_calib_copy", "csgs_calib_atomics", "csgs_calib_mfma_f64", "csgs_calib_lookups"]


class CsgsError(RuntimeError):
    def __init__(self, code, where):
        super().__init__(f"{where}: {strerror(code)} ({code})")
        self.code = code


class Graph(C.Structure):
    """csgs_graph: host struct of device pointers."""
    _fields_ = [("n_nodes", C.c_int64), ("nnz", C.c_int64), ("rowptr", C.c_void_p),
                ("colidx", C.c_void_p), ("val", C.c_void_p), ("local_lo", C.c_int32),
                ("local_hi", C.c_int32), ("rownorm2_max", C.c_float)]


class Workspace(C.Structure):
    """csgs_workspace: host descriptor of the caller-owned scratch buffer."""
    _fields_ = [("base", C.c_void_p), ("bytes", C.c_size_t), ("n_nodes", C.c_int64),
                ("nS_max", C.c_int32), ("B_max", C.c_int32), ("edges_max", C.c_int64), ("rows_buf", C.c_uint64),
                ("has_draw", C.c_uint64), ("draw_B", C.c_int32), ("has_next", C.c_int32),
                ("n_inst", C.c_int32), ("scan_mode", C.c_int32), ("inst_stride", C.c_int64)]


class InstStrides(C.Structure):
    """csgs_inst_strides: byte strides between the instances of the _n compute calls."""
    _fields_ = [("n_inst", C.c_int32), ("reserved", C.c_int32), ("adj", C.c_int64), ("x", C.c_int64),
                ("x_remote", C.c_int64), ("out", C.c_int64)]


class RemoteOut(C.Structure):
    """csgs_remote_out: where csgs_sample_layer leaves the remote split of the new node set."""
    _fields_ = [("local_lo", C.c_int32), ("local_hi", C.c_int32), ("part_bounds", C.c_void_p), ("P", C.c_int32),
                ("remote_total", C.c_void_p), ("per_part", C.c_void_p), ("src_row", C.c_void_p),
                ("remote_ids", C.c_void_p)]


class ProbStats(C.Structure):
    """csgs_prob_stats as laid out on the device (64 bytes)."""
    _fields_ = [("n_cand", C.c_int64), ("n_local", C.c_int64), ("n_remote", C.c_int64),
                ("edges_scanned", C.c_int64), ("w_local", C.c_uint64), ("w_remote", C.c_uint64),
                ("total", C.c_uint64), ("shift", C.c_int32), ("skew_fx", C.c_int32)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is not built; run `python -c 'import __graft_entry__ as g; g.build()'`")
        L = C.CDLL(LIB_PATH)
        vp, i32, i64, u64, u32, f32, sz = (C.c_void_p, C.c_int32, C.c_int64, C.c_uint64, C.c_uint32,
                                           C.c_float, C.c_size_t)
        L.csgs_workspace_bytes.restype = sz
        L.csgs_workspace_bytes.argtypes = [i64, i32, i32, i64]
        L.csgs_workspace_clean_bytes.restype = sz
        L.csgs_workspace_clean_bytes.argtypes = [i64]
        L.csgs_workspace_init.argtypes = [C.POINTER(Workspace), vp]
        L.csgs_workspace_wait_limit.argtypes = [C.POINTER(Workspace), i64, vp]
        L.csgs_fixed_point.argtypes = [i32, f32, f32, C.POINTER(i32), C.POINTER(i64)]
        L.csgs_build_probs.argtypes = [C.POINTER(Graph), vp, i32, vp, f32, vp, vp, vp, vp, i64, vp, C.POINTER(Workspace), vp, vp]
        L.csgs_build_probs_auto.argtypes = [C.POINTER(Graph), vp, i32, vp, f32, i32, f32, vp, vp, vp, vp, i64, vp,
                                            C.POINTER(Workspace), vp, vp]
        L.csgs_sample_layer.argtypes = [C.POINTER(Graph), vp, i32, vp, vp, i64, vp, i32, u64, u64, vp, u32,
                                        vp, vp, vp, vp, vp, vp, vp, i64, vp, C.POINTER(RemoteOut), C.POINTER(Workspace), vp, vp]
        L.csgs_draw_nodes.argtypes = [i64, vp, vp, i64, vp, i32, u64, u64, vp, u32, vp, vp, vp, vp, C.POINTER(Workspace), vp, vp]
        L.csgs_sampled_adjacency.argtypes = [C.POINTER(Graph), vp, i32, vp, vp, vp, vp, i64, vp, C.POINTER(Workspace), vp, vp]
        L.csgs_remote_count.argtypes = [vp, vp, i32, i32, vp, i32, vp, vp, vp, vp, vp]
        L.csgs_aggregate.argtypes = [vp, vp, vp, i32, vp, vp, vp, i64, i64, vp, i64, i64, vp, i32, C.c_int,
                                     C.c_int, vp, i64, vp]
        L.csgs_layer_gemm.argtypes = [vp, i64, i32, vp, i32, vp, i64, i32, vp, i64, vp]
        L.csgs_gather_rows.argtypes = [vp, i64, i64, i32, C.c_int, vp, i64, vp, vp, i64, vp]
        strides = [C.POINTER(InstStrides)]
        L.csgs_aggregate_n.argtypes = strides + L.csgs_aggregate.argtypes
        L.csgs_layer_gemm_n.argtypes = strides + L.csgs_layer_gemm.argtypes
        L.csgs_gather_rows_n.argtypes = strides + L.csgs_gather_rows.argtypes
        fwd = [vp, vp, vp, i32, vp, vp, vp, i64, i64, vp, i64, i64, vp, i32, C.c_int, C.c_int, vp, i64, i32, vp, i64, vp, i64]
        L.csgs_layer_forward.argtypes = fwd + [vp]
        L.csgs_layer_forward_n.argtypes = strides + fwd + [i64, vp]
        L.csgs_layer_forward_supported.argtypes = [i32, C.c_int, i64, i64]
        L.csgs_layer_gemm_grad_w_scratch_bytes.restype = sz
        L.csgs_layer_gemm_grad_w_scratch_bytes.argtypes = [i32, i32, i32]
        L.csgs_layer_gemm_grad_w.argtypes = [vp, i64, vp, i64, i32, vp, i32, i32, vp, i64, vp, sz, vp]
        L.csgs_layer_gemm_grad_w_static.argtypes = [vp, i64, vp, i64, i32, vp, i32, i32, vp, i64, vp]
        L.csgs_layer_gemm_grad_z.argtypes = [vp, i64, i32, vp, i32, vp, i64, i32, vp, i64, vp]
        L.csgs_aggregate_grad_scratch_bytes.restype = sz
        L.csgs_aggregate_grad_scratch_bytes.argtypes = [i32, i64]
        L.csgs_aggregate_grad.argtypes = [vp, vp, vp, i64, i32, vp, i32, vp, vp, i64, i32, vp, i64, vp, i64, vp, sz, vp]
        L.csgs_strerror.restype = C.c_char_p
        L.csgs_strerror.argtypes = [C.c_int]
        L.csgs_calib_copy.argtypes = [vp, vp, sz, vp]
        L.csgs_calib_lookups.argtypes = [vp, sz, sz, vp, sz, vp]
        L.csgs_calib_atomics.argtypes = [vp, sz, sz, vp]
        L.csgs_calib_mfma_f64.argtypes = [vp, sz, i64, i32, vp]
        L.csgs_profile_enable.argtypes = [C.c_int]
        L.csgs_profile_kernel_name.restype = C.c_char_p
        L.csgs_profile_kernel_name.argtypes = [C.c_int]
        L.csgs_profile_collect.argtypes = [C.POINTER(C.c_double), C.POINTER(C.c_int64)]
        L.csgs_profile_samples.argtypes = [C.POINTER(C.c_float), C.POINTER(C.c_int32), i64, C.POINTER(i64)]
        for name in EXPORTS:
            fn = getattr(L, name)
            # without declared argument types ctypes would pass Python integers as 32-bit values, whose
            # upper half is undefined once they travel on the stack into a 64-bit parameter
            assert fn.argtypes is not None or name in ("csgs_profile_kernel_count",), f"{name}: argument types not declared"
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().csgs_strerror(code).decode()


def _ptr(t):
    """Device pointer of a tensor; ctypes objects (a caller's mutable pointer box) pass through."""
    if t is None or isinstance(t, C._SimpleCData):
        return t
    return C.c_void_p(t.data_ptr())


def _stream(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def _chk(rc, where):
    if rc != OK:
        raise CsgsError(rc, where)


class DevicePtr(C.c_void_p):
    """A device pointer whose value may be changed between runs of a Plan: stands for an array of
    `n` elements wherever a wrapper takes a tensor only for its address and element count."""

    def __init__(self, n, value=None):
        super().__init__(value)
        self.n = n

    def numel(self):
        return self.n


class Plan:
    """Library calls with their arguments already marshalled, to be issued again and again: a serving
    or training loop that repeats the same calls on the same buffers pays the Python-side marshalling
    once.  Arguments that change between runs are passed as ctypes boxes (c_uint64, c_void_p ...) whose
    value is read at every run.  Built with `with csgs.record() as plan:` around ordinary wrapper calls
    (nothing is enqueued while recording); `plan.run()` enqueues them."""

    def __init__(self):
        self.calls = []

    def run(self):
        for fn, args, name in self.calls:
            rc = fn(*args)
            if rc != OK:
                raise CsgsError(rc, name)


_recording = None


class record:
    def __enter__(self):
        global _recording
        assert _recording is None, "csgs.record() does not nest"
        _recording = Plan()
        return _recording

    def __exit__(self, *exc):
        global _recording
        _recording = None
        return False


def _call(name, *args):
    fn = getattr(lib(), name)
    if _recording is not None:
        _recording.calls.append((fn, args, name))
        return
    _chk(fn(*args), name)


def make_graph(rowptr, colidx, val, local_lo, local_hi, rownorm2_max=1.0) -> Graph:
    assert rowptr.dtype == torch.int64 and colidx.dtype == torch.int32 and val.dtype == torch.float32
    g = Graph(rowptr.numel() - 1, colidx.numel(), rowptr.data_ptr(), colidx.data_ptr(), val.data_ptr(),
              local_lo, local_hi, rownorm2_max)
    g._keep = (rowptr, colidx, val)
    return g


def csgs_workspace_bytes(n_nodes, nS_max, B_max, edges_max) -> int:
    return int(lib().csgs_workspace_bytes(n_nodes, nS_max, B_max, edges_max))


def csgs_workspace_clean_bytes(n_nodes) -> int:
    return int(lib().csgs_workspace_clean_bytes(n_nodes))


def make_workspace(buf, n_nodes, nS_max, B_max, edges_max, n_inst=1, inst_stride=0, scan_mode=0) -> Workspace:
    """Descriptor for `buf` (a torch tensor of at least n_inst * csgs_workspace_bytes(...) bytes).
    n_inst > 1: calls through it process that many instances, whose arrays lie inst_stride bytes apart."""
    ws = Workspace(buf.data_ptr(), buf.numel() * buf.element_size(), n_nodes, nS_max, B_max, edges_max, 0, 0, 0, 0,
                   n_inst, scan_mode, inst_stride)
    ws._keep = buf
    return ws


def csgs_workspace_init(ws, stream=None):
    _call("csgs_workspace_init", C.byref(ws), _stream(stream))


def csgs_workspace_wait_limit(ws, polls, stream=None):
    _call("csgs_workspace_wait_limit", C.byref(ws), polls, _stream(stream))


def csgs_fixed_point(nS, skew, rownorm2_max=1.0):
    sh, sfx = C.c_int32(0), C.c_int64(0)
    rc = lib().csgs_fixed_point(nS, skew, rownorm2_max, C.byref(sh), C.byref(sfx))
    return rc, sh.value, sfx.value


def _rows(S, nS):
    """Row capacity of a call: the length of S, or nS when S is None (rows = the latest sampled set)."""
    return S.numel() if S is not None else nS


def csgs_build_probs(g, S, skew, cand_id, cand_w, cdf, q, stats, ws, status, stream=None, nS_dev=None, nS=None):
    """nS_dev: device int32 holding the number of rows of S to use (S.numel() is then the capacity).
    S None: rows = the node set of the latest csgs_sample_layer on `ws`; nS = that call's B."""
    _call("csgs_build_probs", C.byref(g), _ptr(S), _rows(S, nS), _ptr(nS_dev), skew, _ptr(cand_id), _ptr(cand_w), _ptr(cdf),
                                _ptr(q), cand_id.numel(), _ptr(stats), C.byref(ws), _ptr(status), _stream(stream))


def csgs_build_probs_auto(g, S, D, B, skew_max, cand_id, cand_w, cdf, q, stats, ws, status, stream=None,
                          nS_dev=None, nS=None):
    _call("csgs_build_probs_auto", C.byref(g), _ptr(S), _rows(S, nS), _ptr(nS_dev), D, B, skew_max, _ptr(cand_id), _ptr(cand_w),
                                     _ptr(cdf), _ptr(q), cand_id.numel(), _ptr(stats), C.byref(ws), _ptr(status),
                                     _stream(stream))


def csgs_sample_layer(g, S, cand_id, cdf, stats, B, seed, it, layer, S_next, mult, p_incl, n_next,
                      adj_rowptr, adj_col, adj_val, adj_nnz, ws, status, stream=None, iter_dev=None, remote=None, nS=None):
    """iter_dev: device uint64 tensor holding the iteration number (then `it` is ignored).
    remote: a RemoteOut (see make_remote_out): also write the remote split of S_next."""
    _call("csgs_sample_layer", C.byref(g), _ptr(S), _rows(S, nS), _ptr(cand_id), _ptr(cdf), cand_id.numel(),
                                 _ptr(stats), B, seed, it, _ptr(iter_dev), layer, _ptr(S_next), _ptr(mult), _ptr(p_incl),
                                 _ptr(n_next), _ptr(adj_rowptr), _ptr(adj_col), _ptr(adj_val), adj_col.numel(),
                                 _ptr(adj_nnz), None if remote is None else C.byref(remote), C.byref(ws), _ptr(status), _stream(stream))


def make_remote_out(local_lo, local_hi, part_bounds, remote_total, per_part=None, src_row=None, remote_ids=None) -> RemoteOut:
    dp = lambda t: None if t is None else t.data_ptr()
    r = RemoteOut(local_lo, local_hi, dp(part_bounds), 0 if part_bounds is None else part_bounds.numel() - 1, dp(remote_total),
                  dp(per_part), dp(src_row), dp(remote_ids))
    r._keep = (part_bounds, remote_total, per_part, src_row, remote_ids)
    return r


def csgs_draw_nodes(n_nodes, cand_id, cdf, stats, B, seed, it, layer, S_next, mult, p_incl, n_next, ws, status,
                    stream=None, iter_dev=None):
    _call("csgs_draw_nodes", n_nodes, _ptr(cand_id), _ptr(cdf), cand_id.numel(), _ptr(stats), B, seed, it, _ptr(iter_dev), layer,
                               _ptr(S_next), _ptr(mult), _ptr(p_incl), _ptr(n_next), C.byref(ws), _ptr(status),
                               _stream(stream))


def csgs_sampled_adjacency(g, rows, adj_rowptr, adj_col, adj_val, adj_nnz, ws, status, stream=None,
                           n_rows_dev=None):
    _call("csgs_sampled_adjacency", C.byref(g), _ptr(rows), rows.numel(), _ptr(n_rows_dev), _ptr(adj_rowptr), _ptr(adj_col),
                                      _ptr(adj_val), adj_col.numel(), _ptr(adj_nnz), C.byref(ws), _ptr(status),
                                      _stream(stream))


def csgs_remote_count(S_next, n_next, local_lo, local_hi, part_bounds, remote_total, per_part=None,
                      src_row=None, remote_ids=None, stream=None):
    P = 0 if part_bounds is None else part_bounds.numel() - 1
    _call("csgs_remote_count", _ptr(S_next), _ptr(n_next), local_lo, local_hi, _ptr(part_bounds), P,
                                 _ptr(remote_total), _ptr(per_part), _ptr(src_row), _ptr(remote_ids),
                                 _stream(stream))


def _inst(inst):
    """Leading arguments of a compute call: the _n form with its strides, or the plain form."""
    return ("_n", (C.byref(inst),)) if inst is not None else ("", ())


def csgs_aggregate(adj_rowptr, adj_col, adj_val, n_next, X_local, X_remote, src_row, relu_on_input, Z,
                   stream=None, nS_dev=None, inst=None):
    """X_* are 2-D float32 tensors or int16/uint16/bfloat16 tensors holding bfloat16 rows.
    inst (InstStrides): several instances per launch; the tensors are instance 0's."""
    suffix, lead = _inst(inst)
    dtype = F32 if X_local.dtype == torch.float32 else BF16
    F = X_local.shape[1]
    rows_r = 0 if X_remote is None else X_remote.shape[0]
    ld_r = 0 if X_remote is None else X_remote.stride(0)
    if X_remote is not None and rows_r == 0:
        X_remote = None
    Xl_ptr = _ptr(X_local) if X_local.shape[0] > 0 else None
    _call("csgs_aggregate" + suffix, *lead, _ptr(adj_rowptr), _ptr(adj_col), _ptr(adj_val), adj_rowptr.numel() - 1,
                              _ptr(nS_dev), _ptr(n_next), Xl_ptr, X_local.stride(0), X_local.shape[0], _ptr(X_remote),
                              ld_r, rows_r, _ptr(src_row), F, dtype, 1 if relu_on_input else 0, _ptr(Z),
                              Z.stride(0), _stream(stream))


def csgs_layer_gemm(Z, W, H, stream=None, M_dev=None, inst=None):
    M, K = Z.shape
    K2, N = W.shape
    assert K == K2 and H.shape == (M, N)
    suffix, lead = _inst(inst)
    _call("csgs_layer_gemm" + suffix, *lead, _ptr(Z), Z.stride(0), M, _ptr(M_dev), K, _ptr(W), W.stride(0), N, _ptr(H), H.stride(0),
                               _stream(stream))


def csgs_layer_forward_supported(X_local, X_remote=None) -> bool:
    """Whether csgs_layer_forward takes input rows of this width, type and layout."""
    dtype = F32 if X_local.dtype == torch.float32 else BF16
    ld_r = 0 if X_remote is None else X_remote.stride(0)
    return bool(lib().csgs_layer_forward_supported(X_local.shape[1], dtype, X_local.stride(0), ld_r))


def csgs_layer_forward(adj_rowptr, adj_col, adj_val, n_next, X_local, X_remote, src_row, relu_on_input, W, H,
                       Z=None, stream=None, nS_dev=None, inst=None, z_stride=0):
    """H = (P~ sigma?(X)) W in one kernel; Z (optional) also receives P~ sigma?(X).  Arguments as csgs_aggregate and
    csgs_layer_gemm; z_stride: bytes between the instances' Z when inst is given."""
    dtype = F32 if X_local.dtype == torch.float32 else BF16
    F_in = X_local.shape[1]
    K2, N = W.shape
    assert K2 == F_in and H.shape == (adj_rowptr.numel() - 1, N)
    rows_r = 0 if X_remote is None else X_remote.shape[0]
    ld_r = 0 if X_remote is None else X_remote.stride(0)
    if X_remote is not None and rows_r == 0:
        X_remote = None
    Xl_ptr = _ptr(X_local) if X_local.shape[0] > 0 else None
    args = (_ptr(adj_rowptr), _ptr(adj_col), _ptr(adj_val), adj_rowptr.numel() - 1, _ptr(nS_dev), _ptr(n_next), Xl_ptr,
            X_local.stride(0), X_local.shape[0], _ptr(X_remote), ld_r, rows_r, _ptr(src_row), F_in, dtype,
            1 if relu_on_input else 0, _ptr(W), W.stride(0), N, _ptr(H), H.stride(0), _ptr(Z), 0 if Z is None else Z.stride(0))
    if inst is not None:
        _call("csgs_layer_forward_n", C.byref(inst), *args, z_stride, _stream(stream))
    else:
        _call("csgs_layer_forward", *args, _stream(stream))


def csgs_layer_gemm_grad_w_scratch_bytes(M, K, N) -> int:
    return int(lib().csgs_layer_gemm_grad_w_scratch_bytes(M, K, N))


def csgs_layer_gemm_grad_w(Z, G, dW, scratch, stream=None, M_dev=None):
    """dW [K x N] = Z^T G; scratch: a tensor of at least csgs_layer_gemm_grad_w_scratch_bytes(M, K, N) bytes."""
    M, K = Z.shape
    M2, N = G.shape
    assert M == M2 and dW.shape == (K, N)
    _call("csgs_layer_gemm_grad_w", _ptr(Z), Z.stride(0), _ptr(G), G.stride(0), M, _ptr(M_dev), K, N, _ptr(dW), dW.stride(0),
          _ptr(scratch), scratch.numel() * scratch.element_size(), _stream(stream))


GRAD_W_STATIC_BYTES = 32 << 20     # CSGS_GRAD_W_STATIC_BYTES


def csgs_layer_gemm_grad_w_static(Z, G, dW, stream=None, M_dev=None):
    """dW [K x N] = Z^T G with the partial sums in the library's own static device buffer (nothing is allocated)."""
    M, K = Z.shape
    M2, N = G.shape
    assert M == M2 and dW.shape == (K, N)
    _call("csgs_layer_gemm_grad_w_static", _ptr(Z), Z.stride(0), _ptr(G), G.stride(0), M, _ptr(M_dev), K, N, _ptr(dW), dW.stride(0),
          _stream(stream))


def csgs_layer_gemm_grad_z(G, W, dZ, stream=None, M_dev=None):
    """dZ [M x K] = G W^T with W [K x N] as in the forward call."""
    M, N = G.shape
    K, N2 = W.shape
    assert N == N2 and dZ.shape == (M, K)
    _call("csgs_layer_gemm_grad_z", _ptr(G), G.stride(0), M, _ptr(M_dev), N, _ptr(W), W.stride(0), K, _ptr(dZ), dZ.stride(0),
          _stream(stream))


def csgs_aggregate_grad_scratch_bytes(n_cols, adj_cap) -> int:
    return int(lib().csgs_aggregate_grad_scratch_bytes(n_cols, adj_cap))


def csgs_aggregate_grad(adj_rowptr, adj_col, adj_val, n_next, dZ, H_prev, dH_prev, scratch, stream=None, nS_dev=None):
    """dH_prev [n_cols x F] = (P~^T dZ) .* [H_prev > 0]; n_cols = dH_prev.shape[0] (capacity), n_next its device count."""
    nS, F = dZ.shape
    n_cols = dH_prev.shape[0]
    assert adj_rowptr.numel() == nS + 1 and dH_prev.shape[1] == F and (H_prev is None or H_prev.shape[1] == F)
    _call("csgs_aggregate_grad", _ptr(adj_rowptr), _ptr(adj_col), _ptr(adj_val), adj_col.numel(), nS, _ptr(nS_dev), n_cols,
          _ptr(n_next), _ptr(dZ), dZ.stride(0), F, _ptr(H_prev), 0 if H_prev is None else H_prev.stride(0), _ptr(dH_prev),
          dH_prev.stride(0), _ptr(scratch), scratch.numel() * scratch.element_size(), _stream(stream))


def csgs_gather_rows(X, ids, n_dev, out, stream=None, inst=None):
    """out[k] = X[ids[k]] for k < *n_dev (device int64; None = all of ids)."""
    assert X.dtype == out.dtype and X.shape[1] == out.shape[1] and out.shape[0] >= ids.numel()
    dtype = F32 if X.dtype == torch.float32 else BF16
    suffix, lead = _inst(inst)
    _call("csgs_gather_rows" + suffix, *lead, _ptr(X), X.stride(0), X.shape[0], X.shape[1], dtype, _ptr(ids), ids.numel(),
                                _ptr(n_dev), _ptr(out), out.stride(0), _stream(stream))


def csgs_profile_enable(on: bool):
    _call("csgs_profile_enable", 1 if on else 0)


def csgs_profile_collect():
    """{kernel name: (summed ms, launches)} since the last collect; call after synchronising."""
    n = lib().csgs_profile_kernel_count()
    ms = (C.c_double * n)()
    cnt = (C.c_int64 * n)()
    _call("csgs_profile_collect", ms, cnt)
    return {lib().csgs_profile_kernel_name(k).decode(): (ms[k], cnt[k]) for k in range(n) if cnt[k]}


def csgs_profile_samples(cap=1 << 16):
    """{kernel name: [ms of every launch]} since the last collect (does not reset); call after synchronising."""
    ms = (C.c_float * cap)()
    kid = (C.c_int32 * cap)()
    n = C.c_int64(0)
    _call("csgs_profile_samples", ms, kid, cap, C.byref(n))
    out = {}
    for i in range(min(cap, n.value)):
        if ms[i] >= 0:
            out.setdefault(lib().csgs_profile_kernel_name(kid[i]).decode(), []).append(ms[i])
    return out


def csgs_calib_copy(dst, src, stream=None):
    nbytes = src.numel() * src.element_size()
    _call("csgs_calib_copy", _ptr(dst), _ptr(src), nbytes, _stream(stream))


def csgs_calib_atomics(table, n_updates, stream=None):
    """n_updates atomic +1 on pseudo-random entries of `table` (an int64 tensor)."""
    _call("csgs_calib_atomics", _ptr(table), table.numel(), n_updates, _stream(stream))


def csgs_calib_lookups(table, n_reads, sink, stream=None):
    """n_reads 8-byte reads of pseudo-random entries of `table` (int64 tensor); sink: int64 tensor of >= 4194304 entries."""
    _call("csgs_calib_lookups", _ptr(table), table.numel(), n_reads, _ptr(sink), sink.numel(), _stream(stream))


CALIB_MFMA_BLOCKS = 2048   # CSGS_CALIB_MFMA_BLOCKS


def csgs_calib_mfma_f64(sink, iters, from_lds=False, stream=None):
    """Matrix-core yardstick; returns the flops of the call.  `sink`: float64 tensor of at least
    CALIB_MFMA_BLOCKS * 256 entries."""
    _call("csgs_calib_mfma_f64", _ptr(sink), sink.numel(), iters, 1 if from_lds else 0, _stream(stream))
    return CALIB_MFMA_BLOCKS * 4 * 64 * 2048 * iters
